// Internal declarations shared by the host API and the kernel launchers.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "curdkv.h"

namespace curdkv {

constexpr int kHeadDim = 128;          // d the kernels are written for
constexpr int kColBlock = 32;          // sketch columns per MFMA tile (M of the 32x32 tile)
constexpr int kMaxColBlocks = 4;       // r padded to 32, 64 or 128
constexpr int kMaxBlocksPerHead = 64;  // partial sums kept per (layer, group)
constexpr int kTileTokens = 32;        // tokens per wave tile
constexpr int kCompactRowsPerBlock = 128;  // output rows per entry of the gather's table of heads
constexpr int kFusedGatherMaxPercent = 11;  // curdkv_compress: share of rows kept up to which the fused kernel also gathers

struct BlockInfo {                     // for gather block b, whose first output row is b*128:
    int64_t head_end;                  //   offsets[head + 1]
    int32_t head;                      //   the head that owns that row
    int32_t pad;
};

// Per-layer state of the head-wise budget allocation (adaptive_kernels.hip), in its workspace.
struct AdaLayerState {
    uint32_t done;                     // workgroups of the layer that have handed in their keys
    uint32_t overflow;                 // some head's cut bin was too full for its segment
    uint32_t pad[2];
};

// Device copy of the offsets, refreshed when they change, followed by the
// per-gather-block table.
struct Plan {
    int64_t* d_offsets = nullptr;      // [heads + 1]
    BlockInfo* d_block_info = nullptr; // [max_blocks]
    char* d_buf = nullptr;             // one allocation holding both
    char* h_staging = nullptr;         // pinned, same layout
    size_t max_blocks = 0;
    std::vector<int64_t> cached;       // what d_offsets holds (after the queued copy)
    bool valid = false;
    hipEvent_t copied = nullptr;       // recorded after the last staging -> device copy
    bool copy_pending = false;
    hipStream_t copy_stream = nullptr; // the stream that copy was queued on
};

}  // namespace curdkv

struct curdkv_ctx {
    curdkv_config cfg;
    int device = 0;
    int heads = 0;                     // layers * kv_heads
    int col_blocks = 0;                // padded sketch_dim / 32 (1, 2 or 4)
    size_t g_elems_per_head = 0;       // packed operand elements per (layer, group)
    void* d_G = nullptr;               // packed sketches, storage type
    float* d_partial = nullptr;        // [heads, kMaxBlocksPerHead]
    int64_t* d_zero_offsets = nullptr; // [heads + 1] zeros: "keep nothing", for the scores-only use of the fused kernel
    void* d_adaptive_ws = nullptr;     // histograms, key segments and per-layer state of the head-wise budget allocation
    curdkv::BlockInfo* d_adaptive_blocks = nullptr;  // gather block table built on the device (curdkv_compress_adaptive)
    float* d_scores_ws = nullptr;      // [heads, max_tokens], allocated when curdkv_compress needs it
    int lds_limit = 0;                 // max dynamic LDS per workgroup, bytes
    int num_cu = 0;
    curdkv::Plan plan;
};

namespace curdkv {

// sketch_host.cpp
void sketch_values(const curdkv_config& cfg, int layer, int head, float* G /*[d*r], rounded*/);
void round_to_storage(float* G, size_t count, int dtype);
// Pack row-major G[d][r] (already rounded) into the A-operand layout of one head.
void pack_sketch(const curdkv_config& cfg, int col_blocks, const float* G, void* packed);
size_t packed_elems(int col_blocks);

// kernel launchers; all return hipGetLastError() after the launch
// normalise = false leaves the un-normalised products in `scores` and the per-block
// sums in ctx->d_partial (*blocks_per_head of them per head) for launch_select to scale.
hipError_t launch_scores(const curdkv_ctx* ctx, const void* K, const void* V, int64_t n,
                         float* scores, hipStream_t stream, bool normalise = true,
                         int* blocks_per_head = nullptr, int64_t out_stride = 0, int64_t out_offset = 0,
                         double* sums = nullptr, bool restart = false, bool* summed = nullptr);
// sums (device, [heads]) given: where one block scores a whole head, the kernel itself adds the
// head's total to sums[head] (after zeroing it if `restart`) and *summed is set; otherwise the
// caller adds the partial sums (launch_accumulate).
hipError_t launch_accumulate(const curdkv_ctx* ctx, int blocks_per_head, double* sums, bool reset,
                             hipStream_t stream);
hipError_t launch_normalise_sums(const curdkv_ctx* ctx, const float* raw, const double* sums,
                                 int64_t stride, int64_t n, float* scores, hipStream_t stream);
hipError_t launch_fold(const curdkv_ctx* ctx, const float* scores_q, int64_t n, float* scores,
                       hipStream_t stream);
// scale_blocks > 0: `scores` holds un-normalised products; the kernel divides them by
// the head's sum (ctx->d_partial, scale_blocks partial sums per head), selects on the
// result and writes it back, which is what normalisation followed by selection gives
// (write_scaled = false: selects on the divided values but leaves `scores` as they are, for
// callers that do not want the scores).
// known_thresholds (device, one {key, need} pair per head as the budget allocation leaves them,
// adaptive_thresholds): heads whose entry is valid skip the search for their threshold.
hipError_t launch_select(const curdkv_ctx* ctx, float* scores, int64_t n, int32_t n_sink,
                         const int64_t* d_offsets, int32_t* indices, hipStream_t stream,
                         int scale_blocks = 0, bool write_scaled = true,
                         const void* known_thresholds = nullptr);
hipError_t launch_compact(const curdkv_ctx* ctx, const void* K, const void* V, int64_t n,
                          const int32_t* indices, const int64_t* d_offsets, int64_t total,
                          void* K_out, void* V_out, hipStream_t stream,
                          const BlockInfo* block_info = nullptr);   // default: the table of the host-side plan
hipError_t configure_kernels(curdkv_ctx* ctx);
hipError_t configure_select(curdkv_ctx* ctx);
hipError_t configure_fused(curdkv_ctx* ctx);
hipError_t configure_adaptive(curdkv_ctx* ctx);
size_t adaptive_workspace_bytes(const curdkv_ctx* ctx);
// workspace: adaptive_workspace_bytes(ctx) bytes of device memory; nothing in it has to be
// cleared beforehand, and its contents mean nothing after the call.
// hist_ready: the per-head histograms (adaptive_hist_buffer) have been written, and the layers'
// state (adaptive_layer_state) reset, by a kernel launched earlier on the stream (launch_fused
// with hist_out); otherwise a kernel of this call makes them from `scores`.
// offsets, block_info (device) given: where budgets are allotted layer-wide, the same launch
// also writes the budgets' prefix sums (every layer keeps kv_heads*k rows) and the gather's
// block table, and *planned is set; where every head gets the same budget they are left to
// launch_adaptive_plan and *planned stays false.
hipError_t launch_adaptive(const curdkv_ctx* ctx, void* workspace, const float* scores, int64_t n, int32_t k,
                           int32_t sp, int32_t g, long long R, int32_t* budgets, hipStream_t stream,
                           bool hist_ready = false, int64_t* offsets = nullptr, BlockInfo* block_info = nullptr,
                           bool* planned = nullptr);
uint32_t* adaptive_hist_buffer(const curdkv_ctx* ctx, void* workspace);
// per head {threshold key, ties to keep} after launch_adaptive has allotted budgets layer-wide
// (key 0xFFFFFFFF where a head's budget comes from its safeguard, not from the layer's threshold)
const void* adaptive_thresholds(const curdkv_ctx* ctx, void* workspace);
AdaLayerState* adaptive_layer_state(const curdkv_ctx* ctx, void* workspace);
// The static device array that serves as that workspace for curdkv_adaptive_budgets_noalloc:
// its address on `device` (looked up by adaptive_static_workspace_init, which curdkv_create
// calls with the device current), and the number of (layer, group) pairs it is sized for.
hipError_t adaptive_static_workspace_init(int device);
void* adaptive_static_workspace(int device);
int adaptive_static_max_heads();
// offsets[i] = budgets[0] + .. + budgets[i-1], kept within [0, total] (offsets[heads] = total), and
// the gather block table for them; everything on the device.
hipError_t launch_adaptive_plan(const curdkv_ctx* ctx, const int32_t* budgets, int64_t n, int64_t total,
                                int64_t* offsets, BlockInfo* block_info, hipStream_t stream);
bool fused_applicable(const curdkv_ctx* ctx, int64_t n);
// hist_out (device, [heads][4096]) given: the kernel also writes every head's histogram of the
// candidates' keys (tokens n_sink and up) over the 4096 bins of the selection (select_device.h)
// and resets layer_state, for the head-wise budget allocation that follows it.
hipError_t launch_fused(const curdkv_ctx* ctx, const void* K, const void* V, int64_t n, int32_t n_sink,
                        const int64_t* d_offsets, float* scores, int32_t* indices, void* K_out,
                        void* V_out, hipStream_t stream, uint32_t* hist_out = nullptr,
                        AdaLayerState* layer_state = nullptr);

}  // namespace curdkv
