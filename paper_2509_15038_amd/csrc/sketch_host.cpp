// Host-side generation of the Gaussian sketch G (the sampling step of Algorithm 1:
// a d x r matrix of independent normal entries with variance 1/r) and its packing
// into the MFMA A-operand layout the scoring kernels read.
//
// The paper fixes no generator.  Each element is addressed by a counter and
// built from two SplitMix64 outputs through Box-Muller, so any (layer, group)
// can be generated on its own and a second implementation can reproduce it.

#include <cmath>
#include <cstring>

#include "curdkv_internal.h"

namespace curdkv {

namespace {

inline uint64_t splitmix64_output(uint64_t seed, uint64_t index) {
    // output number `index` (1-based) of the SplitMix64 stream started at `seed`
    uint64_t z = seed + index * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

inline uint16_t bf16_bits_rne(float x) {
    uint32_t u;
    std::memcpy(&u, &x, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<uint16_t>(u >> 16);
}

inline float bf16_bits_to_float(uint16_t b) {
    uint32_t u = static_cast<uint32_t>(b) << 16;
    float x;
    std::memcpy(&x, &u, 4);
    return x;
}

}  // namespace

void round_to_storage(float* G, size_t count, int dtype) {
    if (dtype != CURDKV_DTYPE_BF16) return;
    for (size_t i = 0; i < count; ++i) G[i] = bf16_bits_to_float(bf16_bits_rne(G[i]));
}

void sketch_values(const curdkv_config& cfg, int layer, int head, float* G) {
    const uint64_t d = static_cast<uint64_t>(cfg.head_dim);
    const uint64_t r = static_cast<uint64_t>(cfg.sketch_dim);
    const uint64_t group = static_cast<uint64_t>(layer) * cfg.kv_heads + head;
    const double two_m53 = 1.0 / 9007199254740992.0;
    const double two_pi = 6.283185307179586476925286766559;
    for (uint64_t i = 0; i < d; ++i) {
        for (uint64_t j = 0; j < r; ++j) {
            const uint64_t c = (group * d + i) * r + j;
            const uint64_t w1 = splitmix64_output(cfg.seed, 2 * c + 1);
            const uint64_t w2 = splitmix64_output(cfg.seed, 2 * c + 2);
            const double u1 = (static_cast<double>(w1 >> 11) + 1.0) * two_m53;  // (0, 1]
            const double u2 = static_cast<double>(w2 >> 11) * two_m53;          // [0, 1)
            const double z = std::sqrt(-2.0 * std::log(u1)) * std::cos(two_pi * u2);
            // the division is written as in the definition (z / sqrt(r)) so that both
            // implementations round the same double
            G[i * r + j] = static_cast<float>(z / std::sqrt(static_cast<double>(r)));
        }
    }
    round_to_storage(G, d * r, cfg.dtype);
}

size_t packed_elems(int col_blocks) { return static_cast<size_t>(col_blocks) * 4096; }

// bf16: the kernel issues, per 16-column block cb and step s (0..3), one
//   mfma_f32_16x16x32_bf16 whose A operand in lane L is the 8 values
//   G[s*32 + (L/16)*8 + e][cb*16 + L%16], e = 0..7  (the token operand of lane L
//   is the 16-byte chunk s*4 + L/16 of token L%16).
// fp32: per 16-column block cb, step s (0..7) and e (0..3) one mfma_f32_16x16x4f32
//   whose A operand in lane L is G[(s*4 + L/16)*4 + e][cb*16 + L%16]  (the token
//   operand of lane L is float e of the 16-byte chunk s*4 + L/16 of token L%16);
//   the four values of a lane for one (cb, s) lie together, so a lane loads them
//   as one 16-byte word.
void pack_sketch(const curdkv_config& cfg, int col_blocks, const float* G, void* packed) {
    const int r = cfg.sketch_dim;
    auto at = [&](int row, int col) -> float { return col < r ? G[row * r + col] : 0.0f; };
    if (cfg.dtype == CURDKV_DTYPE_BF16) {
        uint16_t* out = static_cast<uint16_t*>(packed);
        for (int cb = 0; cb < 2 * col_blocks; ++cb)
            for (int s = 0; s < 4; ++s)
                for (int lane = 0; lane < 64; ++lane)
                    for (int e = 0; e < 8; ++e)
                        out[((cb * 4 + s) * 64 + lane) * 8 + e] =
                            bf16_bits_rne(at(s * 32 + (lane / 16) * 8 + e, cb * 16 + lane % 16));
    } else {
        float* out = static_cast<float*>(packed);
        for (int cb = 0; cb < 2 * col_blocks; ++cb)
            for (int s = 0; s < 8; ++s)
                for (int lane = 0; lane < 64; ++lane)
                    for (int e = 0; e < 4; ++e)
                        out[((cb * 8 + s) * 64 + lane) * 4 + e] = at((s * 4 + lane / 16) * 4 + e, cb * 16 + lane % 16);
    }
}

}  // namespace curdkv
