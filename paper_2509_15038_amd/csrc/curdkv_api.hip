// Host side of the C ABI: argument checks, context lifetime, offsets upload,
// kernel launches.  No arithmetic of the method happens here except the
// generation of the sketch (sketch_host.cpp), which is an input of the kernels.

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>

#include "curdkv_internal.h"

using namespace curdkv;

namespace {

int padded_col_blocks(int r) {
    if (r <= 32) return 1;
    if (r <= 64) return 2;
    return 4;
}

int check_config(const curdkv_config* cfg) {
    if (!cfg) return CURDKV_ERR_INVALID_ARG;
    if (cfg->layers < 1 || cfg->kv_heads < 1 || cfg->group_size < 1 || cfg->max_tokens < 1)
        return CURDKV_ERR_INVALID_ARG;
    if ((int64_t)cfg->layers * cfg->kv_heads > (1 << 24)) return CURDKV_ERR_INVALID_ARG;
    if (cfg->sketch_dim < 1) return CURDKV_ERR_INVALID_ARG;
    if (cfg->dtype != CURDKV_DTYPE_F32 && cfg->dtype != CURDKV_DTYPE_BF16) return CURDKV_ERR_UNSUPPORTED;
    if (cfg->head_dim != kHeadDim) return CURDKV_ERR_UNSUPPORTED;
    if (cfg->sketch_dim > kColBlock * kMaxColBlocks) return CURDKV_ERR_UNSUPPORTED;
    if (cfg->max_tokens > 0x7FFFFFFFLL) return CURDKV_ERR_UNSUPPORTED;   // indices are int32
    if (cfg->score_source < CURDKV_SCORE_KV || cfg->score_source > CURDKV_SCORE_VALUE) return CURDKV_ERR_INVALID_ARG;
    if (cfg->no_projection != 0 && cfg->no_projection != 1) return CURDKV_ERR_INVALID_ARG;
    return CURDKV_OK;
}

size_t storage_bytes(int dtype) { return dtype == CURDKV_DTYPE_BF16 ? 2 : 4; }

// The context's buffers live on the device that was current at curdkv_create.
bool on_own_device(const curdkv_ctx* ctx) {
    int dev = -1;
    return hipGetDevice(&dev) == hipSuccess && dev == ctx->device;
}

// Checks offsets (host) and makes the device copy current on `stream`.
int sync_offsets(curdkv_ctx* ctx, const int64_t* offsets, const int32_t* budgets, int64_t n,
                 hipStream_t stream, int64_t* total) {
    const int heads = ctx->heads;
    if (offsets[0] != 0) return CURDKV_ERR_INVALID_ARG;
    for (int i = 0; i < heads; ++i) {
        const int64_t k = offsets[i + 1] - offsets[i];
        if (k < 0 || k > n) return CURDKV_ERR_INVALID_ARG;
        if (budgets && (int64_t)budgets[i] != k) return CURDKV_ERR_INVALID_ARG;
    }
    *total = offsets[heads];
    Plan& pl = ctx->plan;
    const size_t off_bytes = ((size_t)(heads + 1) * sizeof(int64_t) + 15) & ~(size_t)15;
    const size_t cmp_bytes = (size_t)(heads + 1) * sizeof(int64_t);
    if (pl.valid && std::memcmp(pl.cached.data(), offsets, cmp_bytes) == 0) {
        // same offsets as last time; a caller that moved to another stream must still see the copy
        if (pl.copy_pending && stream != pl.copy_stream) {
            // (a stream under graph capture cannot wait for work outside its graph; callers
            // that capture have run the same call once, and synchronised, beforehand)
            hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
            if (hipStreamIsCapturing(stream, &cs) != hipSuccess) { (void)hipGetLastError(); cs = hipStreamCaptureStatusActive; }
            if (cs == hipStreamCaptureStatusNone && hipStreamWaitEvent(stream, pl.copied, 0) != hipSuccess)
                return CURDKV_ERR_HIP;
        }
        return CURDKV_OK;
    }
    if (pl.copy_pending) {                       // staging buffer may still be being read
        if (hipEventSynchronize(pl.copied) != hipSuccess) return CURDKV_ERR_HIP;
        pl.copy_pending = false;
    }
    std::memcpy(pl.h_staging, offsets, cmp_bytes);
    // head owning the first row of every gather block
    const size_t blocks = (size_t)((*total + kCompactRowsPerBlock - 1) / kCompactRowsPerBlock);
    BlockInfo* bi = reinterpret_cast<BlockInfo*>(pl.h_staging + off_bytes);
    int h = 0;
    for (size_t b = 0; b < blocks; ++b) {
        const int64_t p = (int64_t)b * kCompactRowsPerBlock;
        while (offsets[h + 1] <= p) ++h;
        bi[b].head_end = offsets[h + 1];
        bi[b].head = h;
        bi[b].pad = 0;
    }
    const size_t bytes = off_bytes + blocks * sizeof(BlockInfo);
    pl.valid = false;
    if (hipMemcpyAsync(pl.d_buf, pl.h_staging, bytes, hipMemcpyHostToDevice, stream) != hipSuccess)
        return CURDKV_ERR_HIP;
    if (hipEventRecord(pl.copied, stream) != hipSuccess) return CURDKV_ERR_HIP;
    pl.copy_pending = true;
    pl.copy_stream = stream;
    std::memcpy(pl.cached.data(), offsets, cmp_bytes);
    pl.valid = true;
    return CURDKV_OK;
}

void release(curdkv_ctx* ctx) {
    if (!ctx) return;
    if (ctx->d_G) (void)hipFree(ctx->d_G);
    if (ctx->d_partial) (void)hipFree(ctx->d_partial);
    if (ctx->d_scores_ws) (void)hipFree(ctx->d_scores_ws);
    if (ctx->d_adaptive_ws) (void)hipFree(ctx->d_adaptive_ws);
    if (ctx->d_adaptive_blocks) (void)hipFree(ctx->d_adaptive_blocks);
    if (ctx->d_zero_offsets) (void)hipFree(ctx->d_zero_offsets);
    if (ctx->plan.d_buf) (void)hipFree(ctx->plan.d_buf);
    if (ctx->plan.h_staging) (void)hipHostFree(ctx->plan.h_staging);
    if (ctx->plan.copied) (void)hipEventDestroy(ctx->plan.copied);
    delete ctx;
}

int upload_sketch(curdkv_ctx* ctx, int group, const float* G_rounded) {
    const size_t elems = ctx->g_elems_per_head;
    const size_t bytes = elems * storage_bytes(ctx->cfg.dtype);
    void* packed = std::malloc(bytes);
    if (!packed) return CURDKV_ERR_OOM;
    pack_sketch(ctx->cfg, ctx->col_blocks, G_rounded, packed);
    hipError_t e = hipMemcpy(static_cast<char*>(ctx->d_G) + (size_t)group * bytes, packed, bytes,
                             hipMemcpyHostToDevice);
    std::free(packed);
    return e == hipSuccess ? CURDKV_OK : CURDKV_ERR_HIP;
}

}  // namespace

extern "C" {

const char* curdkv_strerror(int code) {
    switch (code) {
        case CURDKV_OK: return "ok";
        case CURDKV_ERR_INVALID_ARG: return "invalid argument";
        case CURDKV_ERR_UNSUPPORTED: return "unsupported head_dim, sketch_dim, dtype or size";
        case CURDKV_ERR_HIP: return "HIP runtime error";
        case CURDKV_ERR_OOM: return "out of memory";
        case CURDKV_ERR_TOO_LARGE: return "size beyond the fixed workspace of a call that does not allocate";
        default: return "unknown error code";
    }
}

int curdkv_sketch_host(const curdkv_config* cfg, int32_t layer, int32_t head, float* G_host) {
    const int rc = check_config(cfg);
    if (rc != CURDKV_OK) return rc;
    if (!G_host || layer < 0 || layer >= cfg->layers || head < 0 || head >= cfg->kv_heads)
        return CURDKV_ERR_INVALID_ARG;
    sketch_values(*cfg, layer, head, G_host);
    return CURDKV_OK;
}

int curdkv_create(curdkv_ctx** out, const curdkv_config* cfg) {
    if (!out) return CURDKV_ERR_INVALID_ARG;
    const int rc = check_config(cfg);
    if (rc != CURDKV_OK) return rc;
    curdkv_ctx* ctx = new (std::nothrow) curdkv_ctx();
    if (!ctx) return CURDKV_ERR_OOM;
    ctx->cfg = *cfg;
    ctx->heads = cfg->layers * cfg->kv_heads;
    ctx->col_blocks = padded_col_blocks(cfg->sketch_dim);
    ctx->g_elems_per_head = packed_elems(ctx->col_blocks);

    int lds = 0, cus = 0;
    if (hipGetDevice(&ctx->device) != hipSuccess ||
        hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, ctx->device) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, ctx->device) != hipSuccess) {
        release(ctx);
        return CURDKV_ERR_HIP;
    }
    ctx->lds_limit = lds;
    ctx->num_cu = cus > 0 ? cus : 256;
    // address of the static workspace on this device (curdkv_adaptive_budgets_noalloc); a
    // device number beyond the table only makes that one entry point unavailable
    if (adaptive_static_workspace_init(ctx->device) != hipSuccess) (void)hipGetLastError();

    const size_t g_bytes = (size_t)ctx->heads * ctx->g_elems_per_head * storage_bytes(cfg->dtype);
    const size_t off_bytes = ((size_t)(ctx->heads + 1) * sizeof(int64_t) + 15) & ~(size_t)15;
    ctx->plan.max_blocks = ((size_t)ctx->heads * (size_t)cfg->max_tokens + kCompactRowsPerBlock - 1) /
                               kCompactRowsPerBlock + 1;
    const size_t plan_bytes = off_bytes + ctx->plan.max_blocks * sizeof(BlockInfo);
    if (hipMalloc(&ctx->d_G, g_bytes) != hipSuccess ||
        hipMalloc((void**)&ctx->d_partial, (size_t)ctx->heads * kMaxBlocksPerHead * sizeof(float)) != hipSuccess ||
        hipMalloc((void**)&ctx->plan.d_buf, plan_bytes) != hipSuccess ||
        hipHostMalloc((void**)&ctx->plan.h_staging, plan_bytes, hipHostMallocDefault) != hipSuccess) {
        (void)hipGetLastError();
        release(ctx);
        return CURDKV_ERR_OOM;
    }
    // the head-wise budget allocation's workspace and its device-built gather table (a few
    // tens of KB per head): allocated here so that the adaptive calls are kernel launches only
    if (hipMalloc(&ctx->d_adaptive_ws, adaptive_workspace_bytes(ctx)) != hipSuccess ||
        hipMalloc((void**)&ctx->d_adaptive_blocks, ctx->plan.max_blocks * sizeof(BlockInfo)) != hipSuccess) {
        (void)hipGetLastError();
        release(ctx);
        return CURDKV_ERR_OOM;
    }
    if (hipMalloc((void**)&ctx->d_zero_offsets, off_bytes) != hipSuccess ||
        hipMemset(ctx->d_zero_offsets, 0, off_bytes) != hipSuccess) {
        (void)hipGetLastError();
        release(ctx);
        return CURDKV_ERR_OOM;
    }
    ctx->plan.d_offsets = reinterpret_cast<int64_t*>(ctx->plan.d_buf);
    ctx->plan.d_block_info = reinterpret_cast<BlockInfo*>(ctx->plan.d_buf + off_bytes);
    if (hipEventCreateWithFlags(&ctx->plan.copied, hipEventDisableTiming) != hipSuccess) {
        release(ctx);
        return CURDKV_ERR_HIP;
    }
    try {
        ctx->plan.cached.assign((size_t)ctx->heads + 1, 0);
    } catch (...) {
        release(ctx);
        return CURDKV_ERR_OOM;
    }

    float* G = static_cast<float*>(std::malloc((size_t)cfg->head_dim * cfg->sketch_dim * sizeof(float)));
    if (!G) { release(ctx); return CURDKV_ERR_OOM; }
    int err = CURDKV_OK;
    for (int l = 0; l < cfg->layers && err == CURDKV_OK; ++l)
        for (int h = 0; h < cfg->kv_heads && err == CURDKV_OK; ++h) {
            sketch_values(*cfg, l, h, G);
            err = upload_sketch(ctx, l * cfg->kv_heads + h, G);
        }
    std::free(G);
    if (err == CURDKV_OK && (configure_kernels(ctx) != hipSuccess || configure_select(ctx) != hipSuccess ||
                              configure_fused(ctx) != hipSuccess || configure_adaptive(ctx) != hipSuccess))
        err = CURDKV_ERR_HIP;
    if (err != CURDKV_OK) { release(ctx); return err; }
    *out = ctx;
    return CURDKV_OK;
}

int curdkv_destroy(curdkv_ctx* ctx) {
    if (!ctx) return CURDKV_OK;
    const hipError_t e = hipDeviceSynchronize();
    release(ctx);
    return e == hipSuccess ? CURDKV_OK : CURDKV_ERR_HIP;
}

int curdkv_set_sketch(curdkv_ctx* ctx, int32_t layer, int32_t head, const float* G_host) {
    if (!ctx || !G_host) return CURDKV_ERR_INVALID_ARG;
    if (!on_own_device(ctx)) return CURDKV_ERR_INVALID_ARG;
    if (layer < 0 || layer >= ctx->cfg.layers || head < 0 || head >= ctx->cfg.kv_heads)
        return CURDKV_ERR_INVALID_ARG;
    const size_t count = (size_t)ctx->cfg.head_dim * ctx->cfg.sketch_dim;
    float* G = static_cast<float*>(std::malloc(count * sizeof(float)));
    if (!G) return CURDKV_ERR_OOM;
    std::memcpy(G, G_host, count * sizeof(float));
    round_to_storage(G, count, ctx->cfg.dtype);
    if (hipDeviceSynchronize() != hipSuccess) { std::free(G); return CURDKV_ERR_HIP; }
    const int rc = upload_sketch(ctx, layer * ctx->cfg.kv_heads + head, G);
    std::free(G);
    return rc;
}

int curdkv_uses_fused_kernel(const curdkv_ctx* ctx, int64_t n) {
    if (!ctx || n < 1 || n > ctx->cfg.max_tokens) return CURDKV_ERR_INVALID_ARG;
    return fused_applicable(ctx, n) ? 1 : 0;
}

int curdkv_scores(curdkv_ctx* ctx, const void* K, const void* V, int64_t n, float* scores,
                  void* stream) {
    if (!ctx || !K || !V || !scores) return CURDKV_ERR_INVALID_ARG;
    if (!on_own_device(ctx)) return CURDKV_ERR_INVALID_ARG;
    if (n < 1 || n > ctx->cfg.max_tokens) return CURDKV_ERR_INVALID_ARG;
    if (((uintptr_t)K | (uintptr_t)V) & 15u) return CURDKV_ERR_INVALID_ARG;
    // Where the fused kernel applies, its first three phases (one workgroup per head, scores
    // held in LDS, normalised there and written once) beat the scoring + normalisation pair;
    // all-zero offsets make it stop after the scores.
    if (fused_applicable(ctx, n))
        return launch_fused(ctx, K, V, n, 0, ctx->d_zero_offsets, scores, nullptr, nullptr, nullptr,
                            (hipStream_t)stream) == hipSuccess ? CURDKV_OK : CURDKV_ERR_HIP;
    return launch_scores(ctx, K, V, n, scores, (hipStream_t)stream) == hipSuccess ? CURDKV_OK
                                                                                  : CURDKV_ERR_HIP;
}

int curdkv_fold(curdkv_ctx* ctx, const float* scores_q, int64_t n, float* scores, void* stream) {
    if (!ctx || !scores_q || !scores) return CURDKV_ERR_INVALID_ARG;
    if (!on_own_device(ctx)) return CURDKV_ERR_INVALID_ARG;
    if (n < 1 || n > ctx->cfg.max_tokens) return CURDKV_ERR_INVALID_ARG;
    return launch_fold(ctx, scores_q, n, scores, (hipStream_t)stream) == hipSuccess ? CURDKV_OK
                                                                                    : CURDKV_ERR_HIP;
}

int curdkv_select(curdkv_ctx* ctx, const float* scores, int64_t n, const int32_t* budgets,
                  int32_t n_sink, const int64_t* offsets, int32_t* indices, void* stream) {
    if (!ctx || !scores || !budgets || !offsets) return CURDKV_ERR_INVALID_ARG;
    if (!on_own_device(ctx)) return CURDKV_ERR_INVALID_ARG;
    if (n < 1 || n > ctx->cfg.max_tokens || n_sink < 0) return CURDKV_ERR_INVALID_ARG;
    int64_t total = 0;
    const int rc = sync_offsets(ctx, offsets, budgets, n, (hipStream_t)stream, &total);
    if (rc != CURDKV_OK) return rc;
    if (total == 0) return CURDKV_OK;
    if (!indices) return CURDKV_ERR_INVALID_ARG;
    return launch_select(ctx, const_cast<float*>(scores), n, n_sink, ctx->plan.d_offsets, indices, (hipStream_t)stream) == hipSuccess
               ? CURDKV_OK : CURDKV_ERR_HIP;
}

int curdkv_compact(curdkv_ctx* ctx, const void* K, const void* V, int64_t n, const int32_t* indices,
                   const int64_t* offsets, void* K_out, void* V_out, void* stream) {
    if (!ctx || !K || !V || !offsets) return CURDKV_ERR_INVALID_ARG;
    if (!on_own_device(ctx)) return CURDKV_ERR_INVALID_ARG;
    if (n < 1 || n > ctx->cfg.max_tokens) return CURDKV_ERR_INVALID_ARG;
    if (((uintptr_t)K | (uintptr_t)V | (uintptr_t)K_out | (uintptr_t)V_out) & 15u) return CURDKV_ERR_INVALID_ARG;
    int64_t total = 0;
    const int rc = sync_offsets(ctx, offsets, nullptr, n, (hipStream_t)stream, &total);
    if (rc != CURDKV_OK) return rc;
    if (total == 0) return CURDKV_OK;
    if (!indices || !K_out || !V_out) return CURDKV_ERR_INVALID_ARG;
    return launch_compact(ctx, K, V, n, indices, ctx->plan.d_offsets, total, K_out, V_out,
                          (hipStream_t)stream) == hipSuccess ? CURDKV_OK : CURDKV_ERR_HIP;
}

int curdkv_compress(curdkv_ctx* ctx, const void* K, const void* V, int64_t n, const int32_t* budgets,
                    int32_t n_sink, const int64_t* offsets, float* scores, int32_t* indices,
                    void* K_out, void* V_out, void* stream) {
    if (!ctx || !K || !V || !budgets || !offsets) return CURDKV_ERR_INVALID_ARG;
    if (!on_own_device(ctx)) return CURDKV_ERR_INVALID_ARG;
    if (n < 1 || n > ctx->cfg.max_tokens || n_sink < 0) return CURDKV_ERR_INVALID_ARG;
    if (((uintptr_t)K | (uintptr_t)V | (uintptr_t)K_out | (uintptr_t)V_out) & 15u) return CURDKV_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    int64_t total = 0;
    const int rc = sync_offsets(ctx, offsets, budgets, n, st, &total);
    if (rc != CURDKV_OK) return rc;
    if (total > 0 && (!indices || !K_out || !V_out)) return CURDKV_ERR_INVALID_ARG;
    // One kernel for everything when it applies and about a tenth of the rows or fewer are kept.
    // Beyond, the stand-alone gather kernel (many small workgroups, 32 waves per compute unit)
    // moves rows enough faster than the fused kernel's last phase (one long-lived workgroup of 8
    // waves per unit) to pay for two more launches.  Measured at 256 heads of 32768 tokens, one
    // call at keep 5 / 8 / 10 / 12 / 20 / 30 %: fused 783 / 832 / 863 / 897 / 1029 / 1195 us,
    // scoring phases + selection kernel + gather kernel 792 / 832 / 859 / 887 / 993 / 1125 us:
    // level at a tenth (the paper's strongest compression), 4 to 6 % apart from a fifth on.
    const bool fusable = fused_applicable(ctx, n);
    const bool big_gather = total * 100 > (int64_t)ctx->heads * n * kFusedGatherMaxPercent;
    if (fusable && !big_gather)
        return launch_fused(ctx, K, V, n, n_sink, ctx->plan.d_offsets, scores, indices, K_out, V_out, st) == hipSuccess
                   ? CURDKV_OK : CURDKV_ERR_HIP;
    const bool scores_wanted = scores != nullptr;
    if (!scores) {
        if (!ctx->d_scores_ws &&
            hipMalloc((void**)&ctx->d_scores_ws, (size_t)ctx->heads * (size_t)ctx->cfg.max_tokens * sizeof(float)) != hipSuccess) {
            (void)hipGetLastError();
            ctx->d_scores_ws = nullptr;
            return CURDKV_ERR_OOM;
        }
        scores = ctx->d_scores_ws;
    }
    if (fusable) {      // scores from the fused kernel's first phases, then select and gather kernels
        if (launch_fused(ctx, K, V, n, 0, ctx->d_zero_offsets, scores, nullptr, nullptr, nullptr, st) != hipSuccess ||
            launch_select(ctx, scores, n, n_sink, ctx->plan.d_offsets, indices, st) != hipSuccess ||
            launch_compact(ctx, K, V, n, indices, ctx->plan.d_offsets, total, K_out, V_out, st) != hipSuccess)
            return CURDKV_ERR_HIP;
        return CURDKV_OK;
    }
    // the selection kernel normalises on the fly (and writes the normalised scores
    // back), which saves the separate pass over the scores
    int bph = 0;
    if (launch_scores(ctx, K, V, n, scores, st, /*normalise=*/false, &bph) != hipSuccess) return CURDKV_ERR_HIP;
    if (launch_select(ctx, scores, n, n_sink, ctx->plan.d_offsets, indices, st, bph, scores_wanted) != hipSuccess) return CURDKV_ERR_HIP;
    if (total == 0) return CURDKV_OK;
    return launch_compact(ctx, K, V, n, indices, ctx->plan.d_offsets, total, K_out, V_out, st) == hipSuccess
               ? CURDKV_OK : CURDKV_ERR_HIP;
}

int curdkv_adaptive_budgets(curdkv_ctx* ctx, const float* scores, int64_t n, int32_t budget,
                            int32_t n_sink, double alpha, int32_t* budgets_out, void* stream) {
    if (!ctx || !scores || !budgets_out) return CURDKV_ERR_INVALID_ARG;
    if (!on_own_device(ctx)) return CURDKV_ERR_INVALID_ARG;
    if (n < 1 || n > ctx->cfg.max_tokens || n_sink < 0 || budget < 0 || budget > n) return CURDKV_ERR_INVALID_ARG;
    if (!(alpha >= 0.0 && alpha <= 1.0)) return CURDKV_ERR_INVALID_ARG;
    if (ctx->cfg.kv_heads > 1024) return CURDKV_ERR_UNSUPPORTED;
    const int64_t sp = n_sink < n ? n_sink : n;
    int64_t g = (int64_t)std::floor(alpha * (double)budget) - sp;
    if (g < 0) g = 0;
    if (g > n - sp) g = n - sp;
    const long long H = ctx->cfg.kv_heads;
    const long long R = budget > sp ? H * ((long long)budget - sp) - H * g : 0;
    return launch_adaptive(ctx, ctx->d_adaptive_ws, scores, n, budget, (int32_t)sp, (int32_t)g, R, budgets_out,
                           (hipStream_t)stream) == hipSuccess ? CURDKV_OK : CURDKV_ERR_HIP;
}

int curdkv_adaptive_budgets_noalloc(curdkv_ctx* ctx, const float* scores, int64_t n, int32_t budget,
                                    int32_t n_sink, double alpha, int32_t* budgets_out, void* stream) {
    if (!ctx || !scores || !budgets_out) return CURDKV_ERR_INVALID_ARG;
    if (!on_own_device(ctx)) return CURDKV_ERR_INVALID_ARG;
    if (n < 1 || n > ctx->cfg.max_tokens || n_sink < 0 || budget < 0 || budget > n) return CURDKV_ERR_INVALID_ARG;
    if (!(alpha >= 0.0 && alpha <= 1.0)) return CURDKV_ERR_INVALID_ARG;
    if (ctx->cfg.kv_heads > 1024) return CURDKV_ERR_UNSUPPORTED;
    if (ctx->heads > adaptive_static_max_heads()) return CURDKV_ERR_TOO_LARGE;   // beyond the static workspace
    void* ws = adaptive_static_workspace(ctx->device);      // looked up at curdkv_create; nothing is allocated here
    if (!ws) return CURDKV_ERR_HIP;
    const int64_t sp = n_sink < n ? n_sink : n;
    int64_t g = (int64_t)std::floor(alpha * (double)budget) - sp;
    if (g < 0) g = 0;
    if (g > n - sp) g = n - sp;
    const long long H = ctx->cfg.kv_heads;
    const long long R = budget > sp ? H * ((long long)budget - sp) - H * g : 0;
    return launch_adaptive(ctx, ws, scores, n, budget, (int32_t)sp, (int32_t)g, R, budgets_out,
                           (hipStream_t)stream) == hipSuccess ? CURDKV_OK : CURDKV_ERR_HIP;
}

int curdkv_compress_adaptive(curdkv_ctx* ctx, const void* K, const void* V, int64_t n, int32_t budget,
                             int32_t n_sink, double alpha, float* scores, int32_t* budgets_out,
                             int64_t* offsets_out, int32_t* indices, void* K_out, void* V_out, void* stream) {
    if (!ctx || !K || !V || !budgets_out || !offsets_out) return CURDKV_ERR_INVALID_ARG;
    if (!on_own_device(ctx)) return CURDKV_ERR_INVALID_ARG;
    if (n < 1 || n > ctx->cfg.max_tokens || n_sink < 0 || budget < 0 || budget > n) return CURDKV_ERR_INVALID_ARG;
    if (!(alpha >= 0.0 && alpha <= 1.0)) return CURDKV_ERR_INVALID_ARG;
    if (ctx->cfg.kv_heads > 1024) return CURDKV_ERR_UNSUPPORTED;
    if (((uintptr_t)K | (uintptr_t)V | (uintptr_t)K_out | (uintptr_t)V_out) & 15u) return CURDKV_ERR_INVALID_ARG;
    const int64_t total = (int64_t)ctx->heads * budget;       // every layer keeps kv_heads*budget rows
    if (total > 0 && (!indices || !K_out || !V_out)) return CURDKV_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    if (!scores) {
        if (!ctx->d_scores_ws &&
            hipMalloc((void**)&ctx->d_scores_ws, (size_t)ctx->heads * (size_t)ctx->cfg.max_tokens * sizeof(float)) != hipSuccess) {
            (void)hipGetLastError();
            ctx->d_scores_ws = nullptr;
            return CURDKV_ERR_OOM;
        }
        scores = ctx->d_scores_ws;
    }
    // normalised scores first: the allocation compares them across the heads of a layer.  The
    // fused kernel, where it applies, also leaves every head's key histogram in the workspace.
    const bool fused = fused_applicable(ctx, n);
    const hipError_t e = fused
        ? launch_fused(ctx, K, V, n, n_sink, ctx->d_zero_offsets, scores, nullptr, nullptr, nullptr, st,
                       adaptive_hist_buffer(ctx, ctx->d_adaptive_ws), adaptive_layer_state(ctx, ctx->d_adaptive_ws))
        : launch_scores(ctx, K, V, n, scores, st);
    if (e != hipSuccess) return CURDKV_ERR_HIP;
    const int64_t sp = n_sink < n ? n_sink : n;
    int64_t g = (int64_t)std::floor(alpha * (double)budget) - sp;
    if (g < 0) g = 0;
    if (g > n - sp) g = n - sp;
    const long long H = ctx->cfg.kv_heads;
    const long long R = budget > sp ? H * ((long long)budget - sp) - H * g : 0;
    bool planned = false;
    if (launch_adaptive(ctx, ctx->d_adaptive_ws, scores, n, budget, (int32_t)sp, (int32_t)g, R, budgets_out, st,
                        fused, offsets_out, ctx->d_adaptive_blocks, &planned) != hipSuccess)
        return CURDKV_ERR_HIP;
    if (!planned && launch_adaptive_plan(ctx, budgets_out, n, total, offsets_out, ctx->d_adaptive_blocks, st) != hipSuccess)
        return CURDKV_ERR_HIP;
    if (total == 0) return CURDKV_OK;
    // (`planned`: budgets were allotted layer-wide, and the allocation has left every head's threshold)
    if (launch_select(ctx, scores, n, n_sink, offsets_out, indices, st, 0, true,
                      planned ? adaptive_thresholds(ctx, ctx->d_adaptive_ws) : nullptr) != hipSuccess ||
        launch_compact(ctx, K, V, n, indices, offsets_out, total, K_out, V_out, st, ctx->d_adaptive_blocks) != hipSuccess)
        return CURDKV_ERR_HIP;
    return CURDKV_OK;
}

int curdkv_scores_append(curdkv_ctx* ctx, const void* K_new, const void* V_new, int64_t m,
                         int64_t n_old, int64_t stride, float* raw, double* sums, void* stream) {
    if (!ctx || !K_new || !V_new || !raw || !sums) return CURDKV_ERR_INVALID_ARG;
    if (!on_own_device(ctx)) return CURDKV_ERR_INVALID_ARG;
    if (m < 1 || n_old < 0 || stride < 1 || stride > ctx->cfg.max_tokens || m > stride - n_old)
        return CURDKV_ERR_INVALID_ARG;
    if (((uintptr_t)K_new | (uintptr_t)V_new) & 15u) return CURDKV_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)stream;
    int bph = 0;
    bool summed = false;
    if (launch_scores(ctx, K_new, V_new, m, raw, st, /*normalise=*/false, &bph, stride, n_old, sums,
                      n_old == 0, &summed) != hipSuccess)
        return CURDKV_ERR_HIP;
    if (summed) return CURDKV_OK;                 // few new tokens: one launch does it all
    return launch_accumulate(ctx, bph, sums, n_old == 0, st) == hipSuccess ? CURDKV_OK : CURDKV_ERR_HIP;
}

int curdkv_normalise(curdkv_ctx* ctx, const float* raw, const double* sums, int64_t stride,
                     int64_t n, float* scores, void* stream) {
    if (!ctx || !raw || !sums || !scores) return CURDKV_ERR_INVALID_ARG;
    if (!on_own_device(ctx)) return CURDKV_ERR_INVALID_ARG;
    if (n < 1 || stride < n || stride > ctx->cfg.max_tokens) return CURDKV_ERR_INVALID_ARG;
    return launch_normalise_sums(ctx, raw, sums, stride, n, scores, (hipStream_t)stream) == hipSuccess
               ? CURDKV_OK : CURDKV_ERR_HIP;
}

}  // extern "C"
