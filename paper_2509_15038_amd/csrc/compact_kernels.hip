// Gather-compact kernel: the last step of Algorithm 1, which keeps the selected
// rows of the original K_i and V_i, for gfx950.
//
// The packed output is one long list of rows; work is split by output row, not
// by head, so ragged budgets balance by themselves.  A row is copied by a group
// of lanes, 16 bytes per lane, which makes every load and store of a wave cover
// whole rows: 256-byte rows are read at scattered (ascending) addresses and
// written contiguously.  Rows are used once, so loads and stores are marked
// non-temporal.  The head that owns the first row of a stretch of output rows, and
// where that head's rows end, come from a small table the host builds from the
// offsets, so no workgroup has to search and a row address depends on one index
// load only.
//
// Workgroups are many and small: 16 bytes per thread, K and V by different
// workgroups.  Measured on this chip with plain copies of 2 GiB: 16 bytes per thread
// and one array per workgroup 6.45 TB/s, 64 bytes per thread 6.0, 128 bytes 5.7;
// two arrays interleaved in a workgroup 5.9 at best.  This kernel at C3: identity
// indices 6.5 TB/s (was 5.3 with 128 rows of K and V per workgroup), keep 50 %
// 6.26 (was 5.6), keep 10 % 5.97 (was 5.65).

#include "curdkv_internal.h"

namespace curdkv {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// ROW_U4: 16-byte chunks per row (16 for bf16 d=128, 32 for fp32 d=128).
// ITERS: rows a thread copies (all in flight together).  SPLIT: K and V by different workgroups
// (blockIdx.y), else both by the same.  A workgroup covers 256/ROW_U4*ITERS output rows; the
// table of heads has one entry per kCompactRowsPerBlock rows, shared by the workgroups inside.
template <int ROW_U4, int ITERS, bool SPLIT>
__global__ __launch_bounds__(256) void compact_kernel(
    const u32x4* __restrict__ K, const u32x4* __restrict__ V, int64_t n,
    const int32_t* __restrict__ indices, const int64_t* __restrict__ offsets,
    const BlockInfo* __restrict__ block_info, int64_t total, int heads,
    u32x4* __restrict__ K_out, u32x4* __restrict__ V_out) {
    constexpr int kRowsPerIter = 256 / ROW_U4;
    constexpr int kRows = kRowsPerIter * ITERS;
    static_assert(kCompactRowsPerBlock % kRows == 0, "a workgroup's rows lie inside one table entry");
    const int c = threadIdx.x % ROW_U4;
    const int rsub = threadIdx.x / ROW_U4;
    const int64_t p0 = (int64_t)blockIdx.x * kRows;
    const BlockInfo bi = block_info[p0 / kCompactRowsPerBlock];
    int h = bi.head < heads ? (bi.head < 0 ? 0 : bi.head) : heads - 1;   // head of the entry's first row
    int64_t head_end = bi.head_end;                             // offsets[h + 1]
    const u32x4* __restrict__ src = (SPLIT && blockIdx.y) ? V : K;
    u32x4* __restrict__ dst = (SPLIT && blockIdx.y) ? V_out : K_out;

    // index loads first and without branches, so that they are all in flight together
    int32_t idx[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int64_t p = p0 + it * kRowsPerIter + rsub;
        idx[it] = indices[p < total ? p : total - 1];
    }
    size_t row[ITERS];
    bool ok[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int64_t p = p0 + it * kRowsPerIter + rsub;
        // rows ascend: h only moves forward (and never past the last head, whatever the table
        // and the offsets hold: a graph replayed after the context's offsets have changed
        // must not walk off the cache)
        while (head_end <= p && p < total && h + 1 < heads) head_end = offsets[++h + 1];
        ok[it] = p < total && idx[it] >= 0 && idx[it] < n;      // never read outside the cache
        row[it] = ((size_t)h * n + (ok[it] ? idx[it] : 0)) * ROW_U4 + c;
    }
    u32x4 vk[ITERS], vv[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        vk[it] = __builtin_nontemporal_load(src + row[it]);     // row 0 of the head when !ok: in bounds, unused
        if (!SPLIT) vv[it] = __builtin_nontemporal_load(V + row[it]);
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int64_t p = p0 + it * kRowsPerIter + rsub;
        if (ok[it]) {
            __builtin_nontemporal_store(vk[it], dst + (size_t)p * ROW_U4 + c);
            if (!SPLIT) __builtin_nontemporal_store(vv[it], V_out + (size_t)p * ROW_U4 + c);
        }
    }
}

template <int ROW_U4, int ITERS, bool SPLIT>
static void launch_variant(const curdkv_ctx* ctx, const void* K, const void* V, int64_t n, const int32_t* indices,
                           const int64_t* d_offsets, int64_t total, void* K_out, void* V_out, hipStream_t stream,
                           const BlockInfo* block_info) {
    constexpr int kRows = 256 / ROW_U4 * ITERS;
    const int64_t blocks = (total + kRows - 1) / kRows;
    compact_kernel<ROW_U4, ITERS, SPLIT><<<dim3((unsigned)blocks, SPLIT ? 2 : 1), 256, 0, stream>>>(
        (const u32x4*)K, (const u32x4*)V, n, indices, d_offsets, block_info, total, ctx->heads,
        (u32x4*)K_out, (u32x4*)V_out);
}

hipError_t launch_compact(const curdkv_ctx* ctx, const void* K, const void* V, int64_t n,
                          const int32_t* indices, const int64_t* d_offsets, int64_t total,
                          void* K_out, void* V_out, hipStream_t stream, const BlockInfo* block_info) {
    if (total == 0) return hipSuccess;
    if (!block_info) block_info = ctx->plan.d_block_info;
    if (ctx->cfg.dtype == CURDKV_DTYPE_BF16)
        launch_variant<16, 1, true>(ctx, K, V, n, indices, d_offsets, total, K_out, V_out, stream, block_info);
    else
        launch_variant<32, 1, true>(ctx, K, V, n, indices, d_offsets, total, K_out, V_out, stream, block_info);
    return hipGetLastError();
}

}  // namespace curdkv
