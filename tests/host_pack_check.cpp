// Host-only check of the stage planner and the weight packer (csrc/plan.h, csrc/pack.h), meant
// to be built with AddressSanitizer and UndefinedBehaviorSanitizer and run by the CPU test
// suite.  For a sweep of shapes and every weight storage it packs a matrix whose entry
// (col, k) encodes its own position, then walks the packed image the way the kernel's lanes
// do and checks that every (col, k) of the matrix turns up exactly once, at the place the
// plan says, and that everything else is zero.  Also checks e4m3_bits on all 256 codes, the
// row-scaled e4m3 and block-scaled e2m1 forms (exponent rules, rounding, packed codes) and the split of the joint
// output stage into an MFMA part and tail columns.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "pack.h"

using namespace rnnt;

static float e4m3_value(int code)
{
    const int s = code >> 7, e = (code >> 3) & 15, m = code & 7;
    float v = e == 0 ? std::ldexp((float)m, -9) : std::ldexp(1.0f + m / 8.0f, e - 7);
    return s ? -v : v;
}

int main()
{
    long checked = 0;
    // e4m3: every finite code is a fixed point; the two NaN codes and values in between are refused
    for (int code = 0; code < 256; ++code) {
        if ((code & 0x7f) == 0x7f) continue;
        uint8_t back = 0xff;
        if (!e4m3_bits(e4m3_value(code), &back) || back != code) { std::printf("e4m3 code %d\n", code); return 1; }
    }
    uint8_t tmp;
    if (e4m3_bits(0.3f, &tmp) || e4m3_bits(449.0f, &tmp) || e4m3_bits(480.0f, &tmp) ||
        e4m3_bits(1e-9f, &tmp) || e4m3_bits(INFINITY, &tmp) || e4m3_bits(NAN, &tmp)) {
        std::printf("e4m3 accepted a value outside the format\n");
        return 1;
    }
    for (int wt = 0; wt < kWeightTypes; ++wt)
        for (int ts : {1, 3, 8, 32})
            for (int K : {4, 20, 64, 100, 640})
                for (int N : {1, 7, 64, 257, 1030}) {
                    const int ng_all = (N + 3) / 4;
                    auto ng_of = [&](int r) { return range_hi(r, ts, ng_all) - range_lo(r, ts, ng_all); };
                    int gmax = 0;
                    for (int r = 0; r < ts; ++r) gmax = std::max(gmax, ng_of(r));
                    const StagePlan pl = make_stage_plan(K, gmax, wt);
                    // values: small integers that are exact in every storage (e4m3 holds 0..15 exactly)
                    std::vector<float> W((size_t)N * K);
                    static const float mags4[7] = {0.5f, 1.f, 1.5f, 2.f, 3.f, 4.f, 6.f};
                    for (int c = 0; c < N; ++c)
                        for (int k = 0; k < K; ++k)
                            W[(size_t)c * K + k] = pl.kper == 32 ? std::ldexp(mags4[(c * 7 + k * 3) % 7], (c + k / kScaleBlock) % 5 - 2)
                                                                 : (float)(1 + (c * 7 + k * 3) % 15);
                    const std::vector<uint32_t> img = pack_stage(
                        pl, ts, ng_of, [&](int r, int g, int j) -> const float * {
                            const int col = (range_lo(r, ts, ng_all) + g) * 4 + j;
                            return col < N ? W.data() + (size_t)col * K : nullptr;
                        });
                    if (img.size() != (size_t)ts * pl.rank_stride * 4) { std::printf("size\n"); return 1; }
                    std::vector<int> seen((size_t)N * K, 0);
                    for (int rank = 0; rank < ts; ++rank)
                        for (int wave = 0; wave < kWaves; ++wave)
                            for (int slot = 0; slot < pl.slots; ++slot)
                                for (int step = 0; step < pl.nsteps; ++step)
                                    for (int lane = 0; lane < 64; ++lane) {
                                        const uint32_t *q = img.data() + ((size_t)rank * pl.rank_stride +
                                            ((size_t)(wave * pl.slots + slot) * pl.nsteps + step) * 64 + lane) * 4;
                                        const int task = slot * kBlocksPerWg + wave * 16 + (lane >> 2);
                                        const int g = task / pl.nks, ks = task % pl.nks;
                                        const int col = (range_lo(rank, ts, ng_all) + g) * 4 + (lane & 3);
                                        for (int c = 0; c < pl.kper; ++c) {
                                            float v;
                                            if (pl.kper == 4) { std::memcpy(&v, q + c, 4); }
                                            else if (pl.kper == 8) {
                                                const uint32_t bits = ((q[c >> 1] >> (16 * (c & 1))) & 0xffffu) << 16;
                                                std::memcpy(&v, &bits, 4);
                                            } else if (pl.kper == 32) {
                                                // low nibble first; the block's power of two comes from the matrix
                                                const int code = (q[c >> 3] >> (4 * (c & 7))) & 0xf;
                                                const float mag = (code & 7) ? mags4[(code & 7) - 1] : 0.f;
                                                v = (code & 8) ? -mag : mag;
                                                const int kk = (ks * pl.nsteps + step) * pl.kper + c;
                                                if (col < N && kk < K) {
                                                    const int b0 = kk / kScaleBlock * kScaleBlock;
                                                    v = std::ldexp(v, e2m1_block_exponent(W.data() + (size_t)col * K + b0,
                                                                                          std::min(kScaleBlock, K - b0)));
                                                }
                                            } else {
                                                v = e4m3_value((q[c >> 2] >> (8 * (c & 3))) & 0xff);
                                            }
                                            const int k = (ks * pl.nsteps + step) * pl.kper + c;
                                            const bool real_cell = task < ng_of(rank) * pl.nks && col < N && k < K;
                                            if (!real_cell) {
                                                if (v != 0.0f) { std::printf("padding not zero\n"); return 1; }
                                                continue;
                                            }
                                            if (v != W[(size_t)col * K + k]) { std::printf("wrong value\n"); return 1; }
                                            seen[(size_t)col * K + k]++;
                                            ++checked;
                                        }
                                    }
                    for (int v : seen)
                        if (v != 1) { std::printf("wt %d ts %d K %d N %d: a weight appears %d times\n", wt, ts, K, N, v); return 1; }
                }
    // joint output stage: columns beyond a whole number of groups per rank become tail columns
    // when that buys a finer K slicing
    for (int wt = 0; wt < kWeightTypes; ++wt)
        for (int tj : {1, 2, 8, 16, 32})
            for (int J : {64, 320, 640})
                for (int NOUT : {5, 17, 257, 1024, 1025, 1027, 1030, 1033, 4097}) {
                    const JointSplit js = plan_joint_stage(NOUT, J, tj, wt, false);
                    const StagePlan plain = make_stage_plan(J, ((NOUT + 3) / 4 + tj - 1) / tj, wt);
                    const long cost = (long)js.plan.slots * (js.plan.nsteps + kPassOverheadSteps);
                    const long cost_plain = (long)plain.slots * (plain.nsteps + kPassOverheadSteps);
                    bool good = js.nout_m + js.n_tail == NOUT && js.n_tail >= 0 && js.n_tail <= tj;
                    if (js.n_tail > 0)
                        good = good && js.nout_m > 0 && js.nout_m % (4 * tj) == 0 && cost + kTailCostSteps < cost_plain;
                    else
                        good = good && cost == cost_plain;
                    if (!good) { std::printf("joint split NOUT %d J %d tj %d wt %d\n", NOUT, J, tj, wt); return 1; }
                    ++checked;
                }
    {   // the case the split was made for: 1024 labels + blank, eight ranks, fp32
        const JointSplit js = plan_joint_stage(1025, 640, 8, kWeightF32, false);
        if (js.nout_m != 1024 || js.n_tail != 1 || js.plan.nks != 4 || js.plan.nsteps != 40 || js.plan.slots != 1) {
            std::printf("joint split of 1025 columns over 8 ranks: %d + %d, nks %d nsteps %d\n", js.nout_m, js.n_tail,
                        js.plan.nks, js.plan.nsteps);
            return 1;
        }
        const JointSplit even = plan_joint_stage(1024, 640, 8, kWeightF32, false);
        if (even.n_tail != 0 || even.nout_m != 1024) { std::printf("joint split of 1024 columns\n"); return 1; }
    }
    {   // row-scaled e4m3: exponent rule, rounding to the grid, and a packed image whose codes
        // times the row's power of two give the weights back
        const float one[3] = {448.0f, -1.0f, 0.25f}, two[2] = {449.0f, 3.0f}, three[2] = {0.f, 0.f};
        const float four[2] = {224.0f, -7.0f}, five[1] = {1e-45f};
        if (e4m3_row_exponent(one, 3) != 0 || e4m3_row_exponent(two, 2) != 1 || e4m3_row_exponent(three, 2) != 0 ||
            e4m3_row_exponent(four, 2) != -1 || e4m3_row_exponent(five, 1) != -100) {
            std::printf("row exponent\n");
            return 1;
        }
        for (int code = 0; code < 127; ++code) {       // every value is a fixed point; midpoints go to the even code
            const float v = e4m3_value(code);
            if (e4m3_round(v) != v || e4m3_round(-v) != -v) { std::printf("round fixed point %d\n", code); return 1; }
            if (code + 1 < 127) {
                const float mid = 0.5f * (v + e4m3_value(code + 1));
                const float want = e4m3_value((code & 1) ? code + 1 : code);
                if (e4m3_round(mid) != want) { std::printf("round tie %d\n", code); return 1; }
                if (e4m3_round(std::nextafter(mid, 0.f)) != v || e4m3_round(std::nextafter(mid, 1e9f)) != e4m3_value(code + 1)) {
                    std::printf("round next to tie %d\n", code);
                    return 1;
                }
            }
        }
        {   // e2m1: codes, rounding (ties to the even code) and the block exponent
            static const float mags[8] = {0.f, 0.5f, 1.f, 1.5f, 2.f, 3.f, 4.f, 6.f};
            uint8_t code = 0xff;
            for (int c = 0; c < 8; ++c) {
                if (!e2m1_bits(mags[c], &code) || code != c) { std::printf("e2m1 code %d\n", c); return 1; }
                if (c && (!e2m1_bits(-mags[c], &code) || code != (c | 8))) { std::printf("e2m1 code -%d\n", c); return 1; }
                if (e2m1_round(mags[c]) != mags[c]) { std::printf("e2m1 fixed point %d\n", c); return 1; }
                if (c + 1 < 8) {
                    const float mid = 0.5f * (mags[c] + mags[c + 1]);
                    if (e2m1_round(mid) != mags[(c & 1) ? c + 1 : c] || e2m1_round(-mid) != -mags[(c & 1) ? c + 1 : c] ||
                        e2m1_round(std::nextafter(mid, 0.f)) != mags[c] || e2m1_round(std::nextafter(mid, 9.f)) != mags[c + 1]) {
                        std::printf("e2m1 round near %g\n", mid);
                        return 1;
                    }
                }
            }
            if (e2m1_bits(0.25f, &code) || e2m1_bits(5.f, &code) || e2m1_bits(8.f, &code) || e2m1_bits(NAN, &code)) {
                std::printf("e2m1 accepted a value outside the format\n");
                return 1;
            }
            const float a[2] = {6.f, -1.f}, b[2] = {6.5f, 1.f}, c3[2] = {3.f, 0.f}, z[2] = {0.f, 0.f};
            if (e2m1_block_exponent(a, 2) != 0 || e2m1_block_exponent(b, 2) != 1 || e2m1_block_exponent(c3, 2) != -1 ||
                e2m1_block_exponent(z, 2) != 0) {
                std::printf("block exponent\n");
                return 1;
            }
        }
        const int K = 100, N = 37, ts = 3, ng_all = (N + 3) / 4;
        auto ng_of = [&](int r) { return range_hi(r, ts, ng_all) - range_lo(r, ts, ng_all); };
        int gmax = 0;
        for (int r = 0; r < ts; ++r) gmax = std::max(gmax, ng_of(r));
        const StagePlan pl = make_stage_plan(K, gmax, kWeightFp8Bf16Arith);
        std::vector<float> W((size_t)N * K);
        for (int c = 0; c < N; ++c)             // e4m3 values times 2^(c - 20), one entry at the top of the range
            for (int k = 0; k < K; ++k)
                W[(size_t)c * K + k] = std::ldexp(k == c ? 448.0f : e4m3_value((c * 31 + k * 7) % 127), c - 20);
        const std::vector<uint32_t> img = pack_stage(
            pl, ts, ng_of, [&](int r, int g, int j) -> const float * {
                const int col = (range_lo(r, ts, ng_all) + g) * 4 + j;
                return col < N ? W.data() + (size_t)col * K : nullptr;
            }, true);
        for (int rank = 0; rank < ts; ++rank)
            for (int wave = 0; wave < kWaves; ++wave)
                for (int slot = 0; slot < pl.slots; ++slot)
                    for (int step = 0; step < pl.nsteps; ++step)
                        for (int lane = 0; lane < 64; ++lane) {
                            const uint32_t *q = img.data() + ((size_t)rank * pl.rank_stride +
                                ((size_t)(wave * pl.slots + slot) * pl.nsteps + step) * 64 + lane) * 4;
                            const int task = slot * kBlocksPerWg + wave * 16 + (lane >> 2);
                            const int g = task / pl.nks, ks = task % pl.nks;
                            const int col = (range_lo(rank, ts, ng_all) + g) * 4 + (lane & 3);
                            for (int c = 0; c < 16; ++c) {
                                const int k = (ks * pl.nsteps + step) * 16 + c;
                                if (!(task < ng_of(rank) * pl.nks && col < N && k < K)) continue;
                                const float v = std::ldexp(e4m3_value((q[c >> 2] >> (8 * (c & 3))) & 0xff), col - 20);
                                if (v != W[(size_t)col * K + k]) { std::printf("row-scaled value\n"); return 1; }
                                ++checked;
                            }
                        }
    }
    std::printf("ok %ld\n", checked);
    return 0;
}
