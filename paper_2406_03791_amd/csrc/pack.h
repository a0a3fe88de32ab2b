// Host-side repacking of a dense stage's weights into the order the decode kernel streams
// them in (see plan.h for the task decomposition).  No device code and no HIP calls here, so
// that the packer can be built and run under host sanitizers on its own.
#pragma once
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <functional>
#include <vector>

#include "plan.h"

namespace rnnt {

// bf16 code of a float that is exactly representable in bf16 (the engine checks that first).
inline uint16_t bf16_bits(float v)
{
    uint32_t u;
    std::memcpy(&u, &v, sizeof u);
    return (uint16_t)(u >> 16);
}

// OCP e4m3 code (1 sign, 4 exponent bits with bias 7, 3 mantissa bits; no infinities, largest
// finite value 448) of a float, if the float is one of its values.
inline bool e4m3_bits(float v, uint8_t *code)
{
    uint32_t u;
    std::memcpy(&u, &v, sizeof u);
    const uint32_t sign = (u >> 31) << 7, expo = (u >> 23) & 0xffu, mant = u & 0x7fffffu;
    if ((u & 0x7fffffffu) == 0) { *code = (uint8_t)sign; return true; }
    if (expo == 0xffu || expo == 0) return false;           // not finite, or an fp32 subnormal
    const int e = (int)expo - 127;
    if (e >= -6) {                                          // e4m3 normal
        if (e > 8 || (mant & 0xfffffu) != 0) return false;
        const uint32_t m = mant >> 20;
        if (e == 8 && m == 7) return false;                 // that code is NaN
        *code = (uint8_t)(sign | ((uint32_t)(e + 7) << 3) | m);
        return true;
    }
    const float t = std::fabs(v) * 512.0f;                  // e4m3 subnormals are m * 2^-9, m = 1..7
    const int m = (int)t;
    if ((float)m != t || m < 1 || m > 7) return false;
    *code = (uint8_t)(sign | (uint32_t)m);
    return true;
}

// Exponent k of the power-of-two scale of a weight row stored as e4m3 codes with a row scale:
// the smallest k with max|row| * 2^-k <= 448, the largest e4m3 value (0 for a row of zeros),
// kept within +-100 so that the scale and every scaled weight stay normal floats.
// With the smallest such k the row keeps the finest grid it can have without overflow, so a row
// that is representable under any scale is representable under this one.
inline int e4m3_row_exponent(const float *row, int n)
{
    float m = 0.f;
    for (int i = 0; i < n; ++i) {
        const float a = std::fabs(row[i]);
        if (!(a <= m)) m = a;                                 // also picks up a NaN
    }
    if (!(m > 0.f) || !std::isfinite(m)) return 0;
    int k = std::ilogb(m) - 8;                                // m * 2^-k in [256, 512)
    if (std::ldexp(m, -k) > 448.0f) ++k;
    return k < -100 ? -100 : (k > 100 ? 100 : k);
}

// Nearest e4m3 value (ties to the even code) of a finite float of magnitude at most 448.
inline float e4m3_round(float v)
{
    const float a = std::fabs(v);
    if (!(a > 0.f)) return v;
    // spacing of the grid around a: 2^(e-3) in the binade of exponent e >= -6, 2^-9 below
    int e = std::ilogb(a);
    if (e < -6) e = -6;
    const float step = std::ldexp(1.0f, e - 3);
    const float r = std::nearbyint(a / step) * step;          // exact: a / step has at most 24 bits
    return std::copysign(r, v);
}

// OCP e2m1 (4 bits: 1 sign, 2 exponent bits with bias 1, 1 mantissa bit; magnitudes 0, 0.5, 1,
// 1.5, 2, 3, 4, 6) code of a float, if the float is one of its values.
inline bool e2m1_bits(float v, uint8_t *code)
{
    static const float mags[8] = {0.f, 0.5f, 1.f, 1.5f, 2.f, 3.f, 4.f, 6.f};
    const float a = std::fabs(v);
    for (int c = 0; c < 8; ++c)
        if (a == mags[c]) { *code = (uint8_t)(c | (std::signbit(v) ? 8 : 0)); return true; }
    return false;
}

// Nearest e2m1 value (ties to the even code) of a finite float of magnitude at most 6.
inline float e2m1_round(float v)
{
    const float a = std::fabs(v);
    // the grid's spacing is 0.5 below 2, 1 from 2 to 4 and 2 above
    const float step = a < 2.f ? 0.5f : (a < 4.f ? 1.f : 2.f);
    return std::copysign(std::nearbyint(a / step) * step, v);
}

// Exponent k of the power-of-two scale of a block of weights stored as e2m1 codes: the
// smallest k with max|block| * 2^-k <= 6 (0 for zeros), kept within +-100.
inline int e2m1_block_exponent(const float *blk, int n)
{
    float m = 0.f;
    for (int i = 0; i < n; ++i) {
        const float a = std::fabs(blk[i]);
        if (!(a <= m)) m = a;
    }
    if (!(m > 0.f) || !std::isfinite(m)) return 0;
    int k = std::ilogb(m) - 2;                                // m * 2^-k in [4, 8)
    if (std::ldexp(m, -k) > 6.0f) ++k;
    return k < -100 ? -100 : (k > 100 ? 100 : k);
}

// The packed image of one stage: 16 bytes per (rank, wave, slot, step, lane) holding 4 floats,
// 8 bf16 codes, 16 e4m3 codes or 32 e2m1 codes (low nibble first) of consecutive K for the
// output column the lane owns.
//   ngroups(rank)        output groups (of 4 columns) the rank owns
//   row_of(rank, g, j)   the weight row (length plan.K) of column j of the rank's group g, or
//                        nullptr for a column beyond the matrix (stays zero)
//   row_scaled           e4m3 only: the codes are those of row * 2^-k, k = e4m3_row_exponent(row)
//                        (e2m1 codes are always scaled, per block of kScaleBlock K values:
//                        k = e2m1_block_exponent of the block)
inline std::vector<uint32_t> pack_stage(const StagePlan &pl, int ts,
                                        const std::function<int(int)> &ngroups,
                                        const std::function<const float *(int, int, int)> &row_of,
                                        bool row_scaled = false)
{
    std::vector<uint32_t> host((size_t)ts * pl.rank_stride * 4, 0u);
    for (int rank = 0; rank < ts; ++rank) {
        const int ntask = ngroups(rank) * pl.nks;
        for (int slot = 0; slot < pl.slots; ++slot)
            for (int wave = 0; wave < kWaves; ++wave)
                for (int lane = 0; lane < 64; ++lane) {
                    const int task = slot * kBlocksPerWg + wave * 16 + (lane >> 2);
                    if (task >= ntask) continue;
                    const int g = task / pl.nks, ks = task % pl.nks;
                    const float *row = row_of(rank, g, lane & 3);
                    if (!row) continue;
                    const int kexp = (row_scaled && pl.kper == 16) ? e4m3_row_exponent(row, pl.K) : 0;
                    for (int step = 0; step < pl.nsteps; ++step) {
                        uint32_t *dst = host.data() +
                                        ((size_t)rank * pl.rank_stride +
                                         ((size_t)(wave * pl.slots + slot) * pl.nsteps + step) * 64 + lane) * 4;
                        const int k0 = (ks * pl.nsteps + step) * pl.kper;
                        if (pl.kper == 4) {
                            for (int c = 0; c < 4; ++c)
                                if (k0 + c < pl.K) std::memcpy(dst + c, row + k0 + c, 4);
                        } else if (pl.kper == 8) {
                            for (int c = 0; c < 8; ++c)
                                if (k0 + c < pl.K)
                                    dst[c >> 1] |= (uint32_t)bf16_bits(row[k0 + c]) << (16 * (c & 1));
                        } else if (pl.kper == 32) {
                            const int b0 = k0 / kScaleBlock * kScaleBlock;     // a load lies inside one block
                            const int kb = b0 < pl.K ? e2m1_block_exponent(row + b0, std::min(kScaleBlock, pl.K - b0)) : 0;
                            for (int c = 0; c < 32; ++c)
                                if (k0 + c < pl.K) {
                                    uint8_t code = 0;
                                    e2m1_bits(std::ldexp(row[k0 + c], -kb), &code);   // checked when the engine was created
                                    dst[c >> 3] |= (uint32_t)code << (4 * (c & 7));
                                }
                        } else {
                            for (int c = 0; c < 16; ++c)
                                if (k0 + c < pl.K) {
                                    uint8_t code = 0;
                                    e4m3_bits(std::ldexp(row[k0 + c], -kexp), &code);   // checked when the engine was created
                                    dst[c >> 2] |= (uint32_t)code << (8 * (c & 3));
                                }
                        }
                    }
                }
    }
    return host;
}

}  // namespace rnnt
