// Device code of the bf16 scoring pass: the projection, row-norm-squared and
// key-value combination steps of Algorithm 1, for gfx950.  Shared by the stand-alone
// scoring kernel and the fused kernel.
//
// The projection is computed transposed, Y^T = G^T A^T (A = K_i or V_i), with
// mfma_f32_16x16x32_bf16: G^T is the A operand (M = 16 sketch columns), a
// sub-tile of 16 token rows is the B operand (N = 16 tokens).  A wave works
// through a contiguous range of 32-token tiles in pairs (64 tokens); a tile is
// two sub-tiles.  In a sub-tile lane L owns token L%16 and, at MFMA step s
// (0..3), the 16 bytes holding d in [s*32 + (L/16)*8, +8): the four lanes of a
// token read 64 contiguous bytes per load instruction and the wave reads whole
// 256-byte rows over the four steps, which the memory system serves as well as
// a fully coalesced stream.  The accumulator of lane L holds sketch coordinates
// cb*16 + 4*(L/16) + {0..3} of token L%16, so the row-norm squared is a sum in
// the lane plus exchanges between the four 16-lane rows, done with the gfx950
// lane-swap instructions (no LDS round trip).  After the exchange every lane of
// a token holds its score; lane row j keeps the score of sub-tile j of the pair,
// so a pair ends with lane L holding the score of token 64*pair + L.  The
// projected rows never leave registers, and scores go to LDS: a global store
// inside the streaming loop costs several percent of the read bandwidth.
#pragma once

#include <type_traits>

#include "curdkv_internal.h"

namespace curdkv {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

union Chunk {           // 16 bytes of a token row: 8 bf16
    uint4 u;
    bf16x8 v;
};

struct TileRegs {       // one 32-token tile of K and of V as seen by a lane
    Chunk k[2][4];
    Chunk v[2][4];
};

template <int CB>       // CB = padded sketch width / 16
struct SketchRegs {
    bf16x8 g[CB][4];
};

template <int CB>
__device__ __forceinline__ void load_sketch(SketchRegs<CB>& G, const uint4* __restrict__ Gp_head, int lane) {
#pragma unroll
    for (int cb = 0; cb < CB; ++cb)
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            Chunk c;
            c.u = Gp_head[(cb * 4 + s) * 64 + lane];
            G.g[cb][s] = c.v;
        }
}

// a[32..63] <-> b[0..31]
__device__ __forceinline__ void swap_halves(float& a, float& b) {
    const u32x2 r = __builtin_amdgcn_permlane32_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
}
// odd 16-lane rows of a <-> even 16-lane rows of b
__device__ __forceinline__ void swap_rows(float& a, float& b) {
    const u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(a), __float_as_uint(b), false, false);
    a = __uint_as_float(r[0]);
    b = __uint_as_float(r[1]);
}

// lk, lv: per-lane partial sums of a token held by lanes t, t+16, t+32, t+48.
// Returns (sum of the four lk) * (sum of the four lv) in all four lanes.
__device__ __forceinline__ float combine_rows(float lk, float lv) {
    swap_halves(lk, lv);                 // lk = [lk rows 0,1 | lv rows 0,1], lv = [lk rows 2,3 | lv rows 2,3]
    float x = lk + lv;                   // rows: lk0+lk2, lk1+lk3, lv0+lv2, lv1+lv3
    float y = x;
    swap_rows(x, y);                     // x = rows 0,0,2,2 ; y = rows 1,1,3,3
    float z = x + y;                     // rows: LK, LK, LV, LV
    float w = z;
    swap_halves(z, w);                   // z = LK everywhere, w = LV everywhere
    return z * w;
}

// Scores tiles [t_begin, t_end) of one head; the score of token `row` is written
// to lds_rows[row - row0].  t_begin must be even, and t_end even or equal to
// ceil(n/32): tiles are handled in pairs and a missing second tile is taken to
// lie beyond n.  Returns this lane's sum of the scores it wrote.  Kh, Vh: the
// head's rows, 16 chunks of 16 bytes each.  Token and tile numbers are 32-bit
// (n < 2^31) to keep the address arithmetic out of the register budget.
//
// SRC selects the ablation of the appendix ("Ablation Study"): kSrcKV is the
// method itself (product of key and value scores), kSrcK / kSrcV score from one
// tensor only and never load the other.  PROJ = false drops the sketch: the score
// is the squared norm of the stored row (the four lanes of a token hold 32 of its
// 128 elements each), so no MFMA and no G.
constexpr int kSrcKV = 0, kSrcK = 1, kSrcV = 2;

__device__ __forceinline__ float chunk_sum_sq(const Chunk& c, float acc) {
    const uint32_t w[4] = {c.u.x, c.u.y, c.u.z, c.u.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float lo = __uint_as_float(w[i] << 16), hi = __uint_as_float(w[i] & 0xFFFF0000u);
        acc = fmaf(lo, lo, acc);
        acc = fmaf(hi, hi, acc);
    }
    return acc;
}

// Phase of a wave's walk (see scan_tiles): odd multipliers, so that neighbouring heads and
// neighbouring waves of a head start at different offsets.
__device__ __forceinline__ uint32_t scan_phase(int head, int wave_of_head) {
    return (uint32_t)head * 5u + (uint32_t)wave_of_head * 3u;
}

// The walk over tiles [t_begin, t_end) of one wave, shared by the storage types: two tile
// buffers, tiles taken in pairs.
//   load_tile(Tile&, tile, check)   issues the loads of one tile; check = std::true_type clamps
//                                   rows to n - 1 (a ragged last tile), std::false_type is for
//                                   tiles known to lie entirely below n: no clamping, no
//                                   predicate, hence no branch, which keeps the steady-state
//                                   loop one basic block so that the compiler's wait counts let
//                                   loads stay in flight;
//   compute_tile(const Tile&, slot) scores the tile as first (0) or second (1) of its pair;
//   store_pair(tile, check)         puts the pair's 64 scores away (tile = its first tile).
// t_begin must be even, and t_end even or equal to ceil(n/32): a missing second tile is taken
// to lie beyond n.
template <class Tile, class Load, class Compute, class Store>
__device__ __forceinline__ void walk_tiles(int32_t n, int32_t t_begin, int32_t t_end, uint32_t phase,
                                           Load load_tile, Compute compute_tile, Store store_pair) {
    const std::true_type checked;
    const std::false_type unchecked;
    if (t_begin < t_end) {
        Tile ra, rb;
        const int32_t full = n / kTileTokens;                   // tiles with all 32 rows below n
        // The walk starts at tile t_begin + rot and wraps at t_end; rot follows from the caller's
        // phase.  Heads lie a power of two apart in memory, so waves of different heads that walk
        // from the same offset of their ranges keep asking the same memory channels for different
        // rows; started at different offsets they stream 2-3 % faster (measured, 256 heads of
        // 32768 tokens).  Only ranges of whole pairs of whole tiles are rotated, by whole pairs.
        const int32_t len = t_end - t_begin;
        const int32_t rot = (t_end <= full && !(len & 1) && len >= 8) ? (int32_t)(phase % (uint32_t)(len >> 1)) * 2 : 0;
        auto at = [&](int32_t i) -> int32_t { const int32_t t = i + rot; return t >= t_end ? t - len : t; };
        int32_t t = t_begin;
        // both buffers are always filled (a lone tile is simply loaded twice): a
        // conditional load here would make every wait in the loop below pessimistic
        load_tile(ra, at(t), checked);
        load_tile(rb, t + 1 < t_end ? at(t + 1) : at(t), checked);
        const int32_t t_steady = t_end < full ? t_end : full;
        for (; t + 4 <= t_steady; t += 2) {                     // tiles t .. t+3 of the walk are whole
            compute_tile(ra, 0);
            __builtin_amdgcn_sched_barrier(0);
            load_tile(ra, at(t + 2), unchecked);
            __builtin_amdgcn_sched_barrier(0);
            compute_tile(rb, 1);
            __builtin_amdgcn_sched_barrier(0);
            load_tile(rb, at(t + 3), unchecked);
            store_pair(at(t), unchecked);
            __builtin_amdgcn_sched_barrier(0);
        }
        for (; t < t_end; t += 2) {                             // last one or two pairs
            compute_tile(ra, 0);
            if (t + 2 < t_end) load_tile(ra, at(t + 2), checked);
            if (t + 1 < t_end) {
                compute_tile(rb, 1);
                if (t + 3 < t_end) load_tile(rb, at(t + 3), checked);
            }
            store_pair(at(t), checked);                         // an absent second tile lies beyond n
        }
    }
}

template <int CB, int SRC = kSrcKV, bool PROJ = true>
__device__ __forceinline__ float scan_tiles(const SketchRegs<CB>& G, const uint4* __restrict__ Kh,
                                            const uint4* __restrict__ Vh, int32_t n, int32_t t_begin,
                                            int32_t t_end, float* lds_rows, int32_t row0, int lane,
                                            uint32_t phase = 0) {
    const int tok = lane & 15, q = lane >> 4;
    float acc_sum = 0.f;
    float pend = 0.f;                                           // this lane's score of the current pair

    auto load_tile = [&](TileRegs& r, int32_t tile, auto check) {
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
            int32_t row = tile * kTileTokens + t2 * 16 + tok;
            if (decltype(check)::value) row = row < n ? row : n - 1;   // ragged tail: reload the last row
            const size_t off = (size_t)(uint32_t)row * 16 + q;
            const uint4* kp = Kh + off;
            const uint4* vp = Vh + off;
            if (SRC != kSrcV) {
#pragma unroll
                for (int s = 0; s < 4; ++s) r.k[t2][s].u = kp[s * 4];
            }
            if (SRC != kSrcK) {
#pragma unroll
                for (int s = 0; s < 4; ++s) r.v[t2][s].u = vp[s * 4];
            }
        }
    };
    auto compute_tile = [&](const TileRegs& r, int slot) {      // slot: 0 = first tile of the pair
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
            // a tensor that is not scored contributes 1/4 per lane: four lanes make exactly 1
            float lk = SRC == kSrcV ? 0.25f : 0.f, lv = SRC == kSrcK ? 0.25f : 0.f;
            if (PROJ) {
                f32x4 ak[CB], av[CB];
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) { ak[cb] = f32x4{0.f, 0.f, 0.f, 0.f}; av[cb] = f32x4{0.f, 0.f, 0.f, 0.f}; }
#pragma unroll
                for (int s = 0; s < 4; ++s)
#pragma unroll
                    for (int cb = 0; cb < CB; ++cb) {
                        if (SRC != kSrcV)
                            ak[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(G.g[cb][s], r.k[t2][s].v, ak[cb], 0, 0, 0);
                        if (SRC != kSrcK)
                            av[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(G.g[cb][s], r.v[t2][s].v, av[cb], 0, 0, 0);
                    }
#pragma unroll
                for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (SRC != kSrcV) lk = fmaf(ak[cb][e], ak[cb][e], lk);
                        if (SRC != kSrcK) lv = fmaf(av[cb][e], av[cb][e], lv);
                    }
            } else {
#pragma unroll
                for (int s = 0; s < 4; ++s) {
                    if (SRC != kSrcV) lk = chunk_sum_sq(r.k[t2][s], lk);
                    if (SRC != kSrcK) lv = chunk_sum_sq(r.v[t2][s], lv);
                }
            }
            const float lkv = combine_rows(lk, lv);
            pend = (q == slot * 2 + t2) ? lkv : pend;
        }
    };
    auto store_pair = [&](int32_t tile, auto check) {           // lane L holds token tile*32 + L
        const int32_t row = tile * kTileTokens + lane;
        if (!decltype(check)::value || row < n) {
            lds_rows[row - row0] = pend;
            acc_sum += pend;
        }
    };
    walk_tiles<TileRegs>(n, t_begin, t_end, phase, load_tile, compute_tile, store_pair);
    return acc_sum;
}

// ---- fp32 storage -----------------------------------------------------------------------
// The same walk and the same lane roles as above with mfma_f32_16x16x4f32: lane L holds token
// L%16 and, of every 64-byte stretch of its row, the 16 bytes (four floats) number L/16, so a
// load instruction again asks for 64 contiguous bytes per row.  One MFMA takes one of the four
// floats as the token operand; its sketch operand in lane L is
// G[(4*s + L/16)*4 + e][16*cb + L%16] for step s = 0..7 and float e = 0..3.  The sketch lives
// in registers up to 64 columns (32*CB floats per lane) and in LDS beyond (gs: the packed
// sketch as it lies in memory, [cb][s][lane] float4).
struct TileRegsF32 {    // one 32-token tile of K and of V as seen by a lane
    float4 k[2][8];
    float4 v[2][8];
};

template <int CB, bool IN_REGS>
struct SketchF32 {
    float4 g[IN_REGS ? CB : 1][8];
};

template <int CB, bool IN_REGS, int SRC = kSrcKV, bool PROJ = true>
__device__ __forceinline__ float scan_tiles_f32(const SketchF32<CB, IN_REGS>& G, const float4* __restrict__ gs,
                                                const float4* __restrict__ Kh, const float4* __restrict__ Vh,
                                                int32_t n, int32_t t_begin, int32_t t_end, float* lds_rows,
                                                int32_t row0, int lane, uint32_t phase = 0) {
    const int tok = lane & 15, q = lane >> 4;
    float acc_sum = 0.f;
    float pend = 0.f;
    auto load_tile = [&](TileRegsF32& r, int32_t tile, auto check) {
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
            int32_t row = tile * kTileTokens + t2 * 16 + tok;
            if (decltype(check)::value) row = row < n ? row : n - 1;
            const size_t off = (size_t)(uint32_t)row * 32 + q;          // 32 float4 per row
            const float4* kp = Kh + off;
            const float4* vp = Vh + off;
            if (SRC != kSrcV) {
#pragma unroll
                for (int s = 0; s < 8; ++s) r.k[t2][s] = kp[s * 4];
            }
            if (SRC != kSrcK) {
#pragma unroll
                for (int s = 0; s < 8; ++s) r.v[t2][s] = vp[s * 4];
            }
        }
    };
    auto compute_tile = [&](const TileRegsF32& r, int slot) {
#pragma unroll
        for (int t2 = 0; t2 < 2; ++t2) {
            float lk = SRC == kSrcV ? 0.25f : 0.f, lv = SRC == kSrcK ? 0.25f : 0.f;
            // a sketch in LDS is read again for every sub-tile: the lane's offset is made opaque
            // here, or the compiler lifts all of the loads out of the walk and runs out of registers
            int gl = lane;
            if (!IN_REGS) asm volatile("" : "+v"(gl));
            if (!PROJ) {                        // squared norm of the stored row: 32 of its 128 floats per lane
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    if (SRC != kSrcV) {
                        const float4 x = r.k[t2][s];
                        lk = fmaf(x.x, x.x, lk); lk = fmaf(x.y, x.y, lk); lk = fmaf(x.z, x.z, lk); lk = fmaf(x.w, x.w, lk);
                    }
                    if (SRC != kSrcK) {
                        const float4 x = r.v[t2][s];
                        lv = fmaf(x.x, x.x, lv); lv = fmaf(x.y, x.y, lv); lv = fmaf(x.z, x.z, lv); lv = fmaf(x.w, x.w, lv);
                    }
                }
            }
#pragma unroll
            for (int cb = 0; cb < (PROJ ? CB : 0); ++cb) {
                f32x4 ak = f32x4{0.f, 0.f, 0.f, 0.f}, av = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const float4 g = IN_REGS ? G.g[IN_REGS ? cb : 0][s] : gs[(cb * 8 + s) * 64 + gl];
                    if (SRC != kSrcV) {
                        const float4 x = r.k[t2][s];
                        ak = __builtin_amdgcn_mfma_f32_16x16x4f32(g.x, x.x, ak, 0, 0, 0);
                        ak = __builtin_amdgcn_mfma_f32_16x16x4f32(g.y, x.y, ak, 0, 0, 0);
                        ak = __builtin_amdgcn_mfma_f32_16x16x4f32(g.z, x.z, ak, 0, 0, 0);
                        ak = __builtin_amdgcn_mfma_f32_16x16x4f32(g.w, x.w, ak, 0, 0, 0);
                    }
                    if (SRC != kSrcK) {
                        const float4 x = r.v[t2][s];
                        av = __builtin_amdgcn_mfma_f32_16x16x4f32(g.x, x.x, av, 0, 0, 0);
                        av = __builtin_amdgcn_mfma_f32_16x16x4f32(g.y, x.y, av, 0, 0, 0);
                        av = __builtin_amdgcn_mfma_f32_16x16x4f32(g.z, x.z, av, 0, 0, 0);
                        av = __builtin_amdgcn_mfma_f32_16x16x4f32(g.w, x.w, av, 0, 0, 0);
                    }
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    if (SRC != kSrcV) lk = fmaf(ak[e], ak[e], lk);
                    if (SRC != kSrcK) lv = fmaf(av[e], av[e], lv);
                }
            }
            const float lkv = combine_rows(lk, lv);
            pend = (q == slot * 2 + t2) ? lkv : pend;
        }
    };
    auto store_pair = [&](int32_t tile, auto check) {
        const int32_t row = tile * kTileTokens + lane;
        if (!decltype(check)::value || row < n) {
            lds_rows[row - row0] = pend;
            acc_sum += pend;
        }
    };
    walk_tiles<TileRegsF32>(n, t_begin, t_end, phase, load_tile, compute_tile, store_pair);
    return acc_sum;
}

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

}  // namespace curdkv
