// Gather-compact kernel: the last step of Algorithm 1, which keeps the selected
// rows of the original K_i and V_i, for gfx950.
//
// The packed output is one long list of rows; work is split by output row, not
// by head, so ragged budgets balance by themselves.  A row is copied by a group
// of lanes, 16 bytes per lane, which makes every load and store of a wave cover
// whole rows: 256-byte rows are read at scattered (ascending) addresses and
// written contiguously.  Rows are used once, so loads and stores are marked
// non-temporal.  The head that owns the first row of each block, and where that
// head's rows end, come from a small table the host builds from the offsets, so
// no block has to search and a row address depends on one index load only.

#include "curdkv_internal.h"

namespace curdkv {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// ROW_U4: 16-byte chunks per row (16 for bf16 d=128, 32 for fp32 d=128)
template <int ROW_U4>
__global__ __launch_bounds__(256) void compact_kernel(
    const u32x4* __restrict__ K, const u32x4* __restrict__ V, int64_t n,
    const int32_t* __restrict__ indices, const int64_t* __restrict__ offsets,
    const BlockInfo* __restrict__ block_info, int64_t total, int heads,
    u32x4* __restrict__ K_out, u32x4* __restrict__ V_out) {
    constexpr int kRowsPerIter = 256 / ROW_U4;
    constexpr int kIters = 4;                                   // rows in flight per thread
    constexpr int kPasses = kCompactRowsPerBlock / (kRowsPerIter * kIters);
    const int c = threadIdx.x % ROW_U4;
    const int rsub = threadIdx.x / ROW_U4;
    const int64_t p0 = (int64_t)blockIdx.x * kCompactRowsPerBlock;
    const BlockInfo bi = block_info[blockIdx.x];
    int h = bi.head < heads ? (bi.head < 0 ? 0 : bi.head) : heads - 1;   // head of row p0
    int64_t head_end = bi.head_end;                             // offsets[h + 1]

    for (int pass = 0; pass < kPasses; ++pass) {
        // index loads first and without branches, so that they are all in flight together
        int32_t idx[kIters];
#pragma unroll
        for (int it = 0; it < kIters; ++it) {
            const int64_t p = p0 + (pass * kIters + it) * kRowsPerIter + rsub;
            idx[it] = indices[p < total ? p : total - 1];
        }
        const u32x4* src_k[kIters];
        const u32x4* src_v[kIters];
        bool ok[kIters];
#pragma unroll
        for (int it = 0; it < kIters; ++it) {
            const int64_t p = p0 + (pass * kIters + it) * kRowsPerIter + rsub;
            // rows ascend: h only moves forward (and never past the last head, whatever the table
            // and the offsets hold: a graph replayed after the context's offsets have changed
            // must not walk off the cache)
            while (head_end <= p && p < total && h + 1 < heads) head_end = offsets[++h + 1];
            ok[it] = p < total && idx[it] >= 0 && idx[it] < n;  // never read outside the cache
            const size_t row = ((size_t)h * n + (ok[it] ? idx[it] : 0)) * ROW_U4 + c;
            src_k[it] = K + row;
            src_v[it] = V + row;
        }
        u32x4 vk[kIters], vv[kIters];
#pragma unroll
        for (int it = 0; it < kIters; ++it) {
            vk[it] = __builtin_nontemporal_load(src_k[it]);     // row 0 of the head when !ok: in bounds, unused
            vv[it] = __builtin_nontemporal_load(src_v[it]);
        }
#pragma unroll
        for (int it = 0; it < kIters; ++it) {
            const int64_t p = p0 + (pass * kIters + it) * kRowsPerIter + rsub;
            if (ok[it]) {
                __builtin_nontemporal_store(vk[it], K_out + (size_t)p * ROW_U4 + c);
                __builtin_nontemporal_store(vv[it], V_out + (size_t)p * ROW_U4 + c);
            }
        }
    }
}

hipError_t launch_compact(const curdkv_ctx* ctx, const void* K, const void* V, int64_t n,
                          const int32_t* indices, const int64_t* d_offsets, int64_t total,
                          void* K_out, void* V_out, hipStream_t stream, const BlockInfo* block_info) {
    if (total == 0) return hipSuccess;
    if (!block_info) block_info = ctx->plan.d_block_info;
    const int64_t blocks = (total + kCompactRowsPerBlock - 1) / kCompactRowsPerBlock;
    if (ctx->cfg.dtype == CURDKV_DTYPE_BF16) {
        compact_kernel<16><<<dim3((unsigned)blocks), 256, 0, stream>>>(
            (const u32x4*)K, (const u32x4*)V, n, indices, d_offsets, block_info, total, ctx->heads,
            (u32x4*)K_out, (u32x4*)V_out);
    } else {
        compact_kernel<32><<<dim3((unsigned)blocks), 256, 0, stream>>>(
            (const u32x4*)K, (const u32x4*)V, n, indices, d_offsets, block_info, total, ctx->heads,
            (u32x4*)K_out, (u32x4*)V_out);
    }
    return hipGetLastError();
}

}  // namespace curdkv
