// Persistent decode kernel for exact RNN-T / TDT greedy decoding on gfx950: the device code,
// included by the translation unit that instantiates it (decode_inst.hip, compiled once per
// loop nest, row-group count and weight storage).
//
// One launch runs the whole data-dependent double loop of Algorithm 1 (or of
// its label-looping form) on the device.  The work-groups form independent
// teams, whose ranks are spread over the XCDs so that every XCD streams only its
// eighth of the packed weights (see spread_layout in engine.hip); a team owns a
// subset of the utterances and runs the loops for them with its own barrier, so
// no team ever waits for another.  Teams of one utterance have a loop nest of
// their own (kFrameLoopingSingle).  Inside a team every
// dense stage is split over the ranks by output columns and exchanged through
// small global buffers; the loop control (blank mask, symbols_added, not_blank,
// per-utterance frame index) is recomputed identically by every rank from the
// exchanged argmax results, so there is no controller rank.  Label looping adds
// joint groups inside a team: the team runs the prediction network for all its
// rows together, the groups search for the labels of their own rows on their own.
#pragma once
#include "engine.h"

namespace rnnt {
namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

struct Ctl {
    int b[kMaxRows], len[kMaxRows], t[kMaxRows], n[kMaxRows], last[kMaxRows];
    int cnt[kMaxRows], sel[kMaxRows], active[kMaxRows], searching[kMaxRows], mask[kMaxRows];
    int hold_k[kMaxRows], hold_d[kMaxRows];
    int emitted[kMaxRows];         // label looping: the row emitted in the current outer iteration
    float hold_v[kMaxRows], hold_lp[kMaxRows];
    int s_row[kMaxSamples], s_frame[kMaxSamples], s_valid[kMaxSamples];
    int s_pidx[kMaxSamples];       // row of the projected frames (utterance * T + frame) of a valid sample, else -1
    int s_qoff[kMaxSamples];       // where the sample's q row starts (LDS copy or exchange buffer)
    int s_k[kMaxSamples], s_d[kMaxSamples];
    float s_v[kMaxSamples], s_lp[kMaxSamples];   // maximum logit and its log-softmax value
    int R, ns, bar_ok, committed;
    int any[2];                    // Algorithm 1: some row emitted in this inner step (two slots, used in turn)
    int f_any_active, f_need_pred, f_any_searching;   // loop decisions of the control wave
    int st_clamped, st_overflow;   // set to 1 by any thread (same value from all writers)
    int durations[kMaxDur];
};

// The control block of the work-group.  It is a namespace-scope LDS object rather than a
// kernel local passed by reference, so every access is an LDS access by construction.
__shared__ Ctl c;

// Values other work-groups will read go through device-scope atomics so that
// they are written through to, and read from, the level all XCDs share.
__device__ __forceinline__ void xstore(float *p, float v)
{
    __hip_atomic_store(reinterpret_cast<unsigned *>(p), __float_as_uint(v), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float xload(const float *p)
{
    return __uint_as_float(__hip_atomic_load(reinterpret_cast<const unsigned *>(p),
                                             __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}
__device__ __forceinline__ void xstore64(unsigned long long *p, unsigned long long v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned long long xload64(const unsigned long long *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// bfloat16 mode: a value that enters a product is rounded to the nearest bfloat16 value (ties to
// even; NaN and infinities pass through) and kept as a float; other modes leave it alone.
template <int WT>
__device__ __forceinline__ float as_operand(float v)
{
    if (!is_bf16_arith(WT)) return v;
    unsigned u = __float_as_uint(v);
    if ((u & 0x7f800000u) != 0x7f800000u) { u += 0x7fffu + ((u >> 16) & 1u); u &= 0xffff0000u; }
    return __uint_as_float(u);
}

// Activation rows in LDS.  In the bfloat16 mode a row holds bf16 values (two bytes each, in K
// order, at the start of the row's storage) and feeds the bf16 MFMA directly; in the other
// modes it holds floats.  `row` is the row's first float slot in either case.
template <int WT>
__device__ __forceinline__ void x_store(float *row, int k, float v)
{
    if (is_bf16_arith(WT))
        reinterpret_cast<unsigned short *>(row)[k] = (unsigned short)(__float_as_uint(as_operand<WT>(v)) >> 16);
    else
        row[k] = v;
}
template <int WT>
__device__ __forceinline__ void x_store2(float *row, int k, float2 v)      // k even
{
    if (is_bf16_arith(WT)) {
        const unsigned lo = __float_as_uint(as_operand<WT>(v.x)) >> 16, hi = __float_as_uint(as_operand<WT>(v.y)) & 0xffff0000u;
        reinterpret_cast<unsigned *>(row)[k >> 1] = lo | hi;
    } else {
        *reinterpret_cast<float2 *>(row + k) = v;
    }
}
template <int WT>
__device__ __forceinline__ void x_store4(float *row, int k, float4 v)      // k a multiple of 4
{
    if (is_bf16_arith(WT)) {
        const unsigned a = (__float_as_uint(as_operand<WT>(v.x)) >> 16) | (__float_as_uint(as_operand<WT>(v.y)) & 0xffff0000u);
        const unsigned b = (__float_as_uint(as_operand<WT>(v.z)) >> 16) | (__float_as_uint(as_operand<WT>(v.w)) & 0xffff0000u);
        *reinterpret_cast<uint2 *>(reinterpret_cast<unsigned *>(row) + (k >> 1)) = make_uint2(a, b);
    } else {
        *reinterpret_cast<float4 *>(row + k) = v;
    }
}

// four consecutive values of an activation row, as floats
template <int WT>
__device__ __forceinline__ float4 x_load4(const float *row, int k)        // k a multiple of 4
{
    if (is_bf16_arith(WT)) {
        const uint2 v = *reinterpret_cast<const uint2 *>(reinterpret_cast<const unsigned *>(row) + (k >> 1));
        return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u),
                           __uint_as_float(v.y << 16), __uint_as_float(v.y & 0xffff0000u));
    }
    return *reinterpret_cast<const float4 *>(row + k);
}

// two e4m3 codes (the low or the high half of `word`) as one word of two bf16, first code in
// the low half; v_cvt_scalef32_pk_bf16_fp8.  The instruction multiplies by the power of two
// that `scale` has as its exponent (its mantissa is ignored): with scale 1 every e4m3 value
// comes out as the bf16 value it is, with the scale of a weight row as that value times the
// row's power of two, still without rounding.
typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
template <bool HIGH>
__device__ __forceinline__ float e4m3x2_to_bf16x2(unsigned word, float scale)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(word, scale, HIGH));
}

// Two e2m1 codes (byte BYTE of `word`, low nibble first) as two bf16 in one 32-bit register,
// times the power of two of `scale`: v_cvt_scalef32_pk_bf16_fp4.
template <int BYTE>
__device__ __forceinline__ float e2m1x2_to_bf16x2(unsigned word, float scale)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(word, scale, BYTE));
}

// Exponent byte of a power-of-two scale (all the widening instructions use of it).
__device__ __forceinline__ unsigned char scale_byte(float scale)
{
    return (unsigned char)((__float_as_uint(scale) >> 23) & 0xffu);
}

typedef short v4s __attribute__((ext_vector_type(4)));
// four bf16 values held in two 32-bit registers, as the operand type of the bf16 MFMA
__device__ __forceinline__ v4s bf16x4(float lo, float hi)
{
    struct { float a, b; } t = {lo, hi};
    return __builtin_bit_cast(v4s, t);
}

// Read-modify-write atomics are issued on pointers typed as global memory: on a generic
// pointer the compiler has to add a run-time test for the private aperture.
typedef __attribute__((address_space(1))) unsigned global_u32;
typedef __attribute__((address_space(1))) int global_i32;
__device__ __forceinline__ global_u32 *as_global(unsigned *p) { return (global_u32 *)p; }
__device__ __forceinline__ global_i32 *as_global(int *p) { return (global_i32 *)p; }

// The thread's index as a value the compiler cannot trace back to the start of the kernel.
// Everything derived from it (row and column numbers, addresses into the exchange buffers and
// LDS) is then computed where it is used; otherwise those loop-invariant values are all
// computed once before the decode loop and kept for its whole length, which takes more
// registers than there are and puts reloads in front of the loads a step waits for.
__device__ __forceinline__ int rederive(int v)
{
    asm volatile("" : "+v"(v));
    return v;
}

struct Wg {
    int team, rank, tid, lane, wave;
    int jg, jrank;       // joint group inside the team and rank inside that group
};

// Synchronisation counters of the work-group (uniform over its threads).
struct Sync {
    unsigned epoch;      // team barriers passed
    unsigned jepoch;     // joint steps taken by the team: tags the exchanged argmax partials
    unsigned pepoch;     // prediction steps taken by the team: tags the exchanged hidden vectors
    long long polls;
};

// Phase timers (100 MHz wall clock), compiled in only for profiling builds.
#ifdef RNNT_PROFILE
__shared__ long long g_prof[24];
__shared__ long long g_prof_last;
#define PROF_MARK(w, slot) do { if ((w).tid == 0) { long long t_ = wall_clock64(); g_prof[slot] += t_ - g_prof_last; g_prof_last = t_; } } while (0)
#else
#define PROF_MARK(w, slot) do { } while (0)
#endif

// Wait until this wave's own loads and stores have been performed.  Exchange
// data is written with device-scope atomic stores (written through to the level
// all XCDs share), so once they are acknowledged nothing has to be flushed: the
// barrier needs no cache write-back or invalidate, which on this part cost tens
// of microseconds per barrier.  The asm is also a compiler barrier for memory.
__device__ __forceinline__ void wait_own_memory_ops()
{
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
}

// Team barrier with a bounded wait.  Returns false when the wait expired or
// another work-group raised the abort flag; the caller then leaves the kernel.
// Ordering: every thread completes its exchange stores, the work-group meets,
// thread 0 announces arrival with a relaxed device-scope add and polls the
// counter; data is read afterwards with device-scope atomic loads only.
__device__ __forceinline__ bool team_barrier(const DecodeParams &p, const Wg &w, Sync &sy)
{
    wait_own_memory_ops();
    __syncthreads();
    sy.epoch += 1;
    if (w.tid == 0) {
        unsigned *ctr = p.bar + w.team * 32;
        const unsigned target = sy.epoch * (unsigned)p.team_size;
        __hip_atomic_fetch_add(as_global(ctr), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        unsigned spins = 0;
        int ok = 1;
        while (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
            ++spins;
            if ((spins & 127u) == 0 &&
                __hip_atomic_load(p.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                ok = 0;
                break;
            }
            if (spins > p.spin_limit) {
                __hip_atomic_store(p.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                ok = 0;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        sy.polls += spins;
        c.bar_ok = ok;
    }
    __syncthreads();
    return c.bar_ok != 0;
}

// The packed weights of a stage are a fixed stream per lane, independent of the
// data, so their loads can start before the stage's input is there: kAhead
// batches of kStepUnroll float4 steps are kept in flight in registers.  Three batches measured
// 1-2 % faster than two on MI355X and four slower again (registers; and a wave's loads return in
// order, so the exchange loads behind a longer window wait longer).  Non-temporal loads
// measured slower: the teams of an XCD profit from each other's L2 lines.
constexpr int kAhead = 3;

struct WeightStream {
    const float4 *base;   // this wave's run of the current pass (uniform over the wave)
    int lane_off;         // the lane's float4 inside a step's 64
    int task;
    float4 q[kAhead][kStepUnroll];
};

// Start the weight stream of a stage for this wave: the first kAhead batches go out.  Every
// lane loads, also one without a task: it reads along with lane (lane & 3) of the wave's first
// block, which costs no extra traffic, and its products are never stored.  That keeps the
// loads free of per-lane conditions.  The packed buffers end in a few steps of padding, so a
// short stage's second batch may read past its last step.
__device__ __forceinline__ void stream_begin(WeightStream &ws, const StageDev &sd, const Wg &w,
                                             int rank, int n_tasks)
{
    // a wave's passes ("slots") follow each other in memory, so its whole stage is one
    // contiguous run of slots * nsteps loads per lane
    ws.task = w.wave * 16 + (w.lane >> 2);
    ws.lane_off = ws.task < n_tasks ? w.lane : (w.lane & 3);
    ws.base = sd.w + (long long)rank * sd.rank_stride + ((long long)(w.wave * sd.slots) * sd.nsteps) * 64;
#pragma unroll
    for (int a = 0; a < kAhead; ++a)
#pragma unroll
        for (int u = 0; u < kStepUnroll; ++u)
            ws.q[a][u] = ws.base[ws.lane_off + (a * kStepUnroll + u) * 64];
}

// One dense stage for this rank:  red[task][rg][col][row] = sum over the task's
// K slice of x[row][k] * W[col][k], rows in groups of 4 (RG groups).
//   ws           weight stream of slot 0, begun by the caller
//   x            LDS, rows `xstride` floats apart; input vector `inp` of a group
//                starts `x_inp_stride` floats further (inp = group / groups_per_inp)
//   red_aliases_x  the results overwrite x (only valid with a single slot)
// WT: how the packed weights are stored.  kWeightF32: a load carries four weights.
// kWeightBf16: a load carries eight bf16 weights, used as two part-steps of four; a bf16
// weight becomes its fp32 value by a shift, the products and sums are fp32 as before.
// kWeightFp8: sixteen e4m3 weights, four part-steps; one conversion instruction widens two.
//   bias         LDS, the rank's slice of the stage's bias vector (4 per group), or nullptr:
//                the accumulators of a group's first K slice start from it, as the sum the
//                oracle forms does
//   scale        kWeightFp8Bf16Arith: LDS, the power of two of each of the rank's weight rows
//                (4 per group), kept as the exponent byte of that float; a lane's weights all
//                belong to one row.  kWeightFp4Bf16Arith: [row][block], one per kScaleBlock K
//                values of the padded row, which is one batch of a lane's loads
template <int RG, int WT>
__device__ __forceinline__ void run_stage(const StageDev &sd, const Wg &w, int n_tasks,
                                          WeightStream &ws, const float *x, int xstride,
                                          int x_inp_stride, int groups_per_inp, float *red,
                                          bool red_aliases_x, const unsigned char *scale,
                                          const float *bias = nullptr)
{
    static_assert(kMaxSamples <= 64, "the samples of a joint step are set up by one wave");
    const int r4 = w.lane & 3;
    // The loads run through the passes without a break (a lane without a task in a pass reads
    // the zero padding of the packed weights), so the pipeline is never empty between passes.
    int left = sd.slots * sd.nsteps;                 // loads from the start of this pass to the end
    for (int slot = 0; slot < sd.slots; ++slot) {
        const int task = ws.task;
        const bool live = task < n_tasks;
        const int g = live ? task / sd.nks : 0;
        const int ks = live ? task - g * sd.nks : 0;
        constexpr int KPER = k_per_load(WT);
        // bfloat16 mode: the activation rows hold bf16, 16 bytes of a row match the 16 bytes (eight
        // weights) of a load, and one load feeds two 4x4x4 bf16 MFMAs; otherwise a load is used
        // in part-steps of four K values on the fp32 4x4x1 MFMA
        // (with e4m3 storage a load carries sixteen weights: two such halves, each widened first)
        constexpr bool BF = is_bf16_arith(WT);
        constexpr int HALVES = BF ? KPER / 8 : KPER / 4;
        const float *xr = x + (g / groups_per_inp) * x_inp_stride + r4 * xstride + ks * sd.nsteps * (BF ? KPER / 2 : KPER);
        // lane r4 of a block accumulates output column r4 of the group for the block's four rows
        const float b0 = (bias && live && ks == 0) ? bias[g * 4 + r4] : 0.f;
        float sc = 1.0f;
        if (WT == kWeightFp8Bf16Arith && live) sc = __uint_as_float((unsigned)scale[g * 4 + r4] << 23);
        // 4-bit codes: this task's run of block scales
        const unsigned char *scp = scale;
        if (WT == kWeightFp4Bf16Arith)
            scp = scale + (g * 4 + r4) * (sd.nks * (sd.nsteps / kStepUnroll)) + ks * (sd.nsteps / kStepUnroll);
        v4f acc[RG];
#pragma unroll
        for (int rg = 0; rg < RG; ++rg) acc[rg] = (v4f){b0, b0, b0, b0};
        // activations of the step after the current one are fetched from LDS while the
        // current step's MFMAs issue; the scheduling barriers keep the compiler from
        // hoisting more LDS reads than that (they would occupy hundreds of registers)
        float4 xa[RG], xb[RG];
#pragma unroll
        for (int rg = 0; rg < RG; ++rg)
            xa[rg] = *reinterpret_cast<const float4 *>(xr + rg * 4 * xstride);
        // Each pass of the loop consumes the kAhead batches in turn and refills a batch in
        // place as soon as it has been used, so the stream needs no register moves.
#pragma unroll 1
        for (int i0 = 0; i0 < sd.nsteps; i0 += kAhead * kStepUnroll) {
#pragma unroll
            for (int a = 0; a < kAhead; ++a) {
                const int i = i0 + a * kStepUnroll;
                if (i < sd.nsteps) {
                    if (WT == kWeightFp4Bf16Arith) sc = live ? __uint_as_float((unsigned)scp[i / kStepUnroll] << 23) : 1.0f;
#pragma unroll
                    for (int u = 0; u < kStepUnroll; ++u) {
                        const float4 raw = ws.q[a][u];
#pragma unroll
                        for (int h = 0; h < HALVES; ++h) {
                            // the row is 4 floats longer than kpad, so the read past the
                            // last step stays inside it
#pragma unroll
                            for (int rg = 0; rg < RG; ++rg)
                                xb[rg] = *reinterpret_cast<const float4 *>(
                                    xr + rg * 4 * xstride + ((i + u) * HALVES + h + 1) * 4);
                            if (BF) {
                                // eight weights of this half as four words of two bf16 each
                                float w0, w1, w2, w3;
                                if (WT == kWeightFp8Bf16Arith) {
                                    // one instruction widens two e4m3 codes to two bf16 and applies the
                                    // row's power of two (nothing is rounded)
                                    const unsigned lo_word = __float_as_uint(h == 0 ? raw.x : raw.z);
                                    const unsigned hi_word = __float_as_uint(h == 0 ? raw.y : raw.w);
                                    w0 = e4m3x2_to_bf16x2<false>(lo_word, sc); w1 = e4m3x2_to_bf16x2<true>(lo_word, sc);
                                    w2 = e4m3x2_to_bf16x2<false>(hi_word, sc); w3 = e4m3x2_to_bf16x2<true>(hi_word, sc);
                                } else if (WT == kWeightFp4Bf16Arith) {
                                    // a word holds the eight codes of this half; one instruction widens
                                    // the two of a byte and applies the block's power of two
                                    const unsigned word = __float_as_uint(h == 0 ? raw.x : (h == 1 ? raw.y : (h == 2 ? raw.z : raw.w)));
                                    w0 = e2m1x2_to_bf16x2<0>(word, sc); w1 = e2m1x2_to_bf16x2<1>(word, sc);
                                    w2 = e2m1x2_to_bf16x2<2>(word, sc); w3 = e2m1x2_to_bf16x2<3>(word, sc);
                                } else {
                                    w0 = raw.x; w1 = raw.y; w2 = raw.z; w3 = raw.w;
                                }
#pragma unroll
                                for (int rg = 0; rg < RG; ++rg) {
                                    acc[rg] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(bf16x4(xa[rg].x, xa[rg].y), bf16x4(w0, w1), acc[rg], 0, 0, 0);
                                    acc[rg] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(bf16x4(xa[rg].z, xa[rg].w), bf16x4(w2, w3), acc[rg], 0, 0, 0);
                                }
#pragma unroll
                                for (int rg = 0; rg < RG; ++rg) xa[rg] = xb[rg];
                                __builtin_amdgcn_sched_barrier(0);
                                continue;
                            }
                            float4 wv;
                            if (WT == kWeightBf16) {
                                const unsigned lo = __float_as_uint(h == 0 ? raw.x : raw.z);
                                const unsigned hi = __float_as_uint(h == 0 ? raw.y : raw.w);
                                wv = make_float4(__uint_as_float(lo << 16), __uint_as_float(lo & 0xffff0000u),
                                                 __uint_as_float(hi << 16), __uint_as_float(hi & 0xffff0000u));
                            } else if (WT == kWeightFp8) {
                                const int word = (int)__float_as_uint(h == 0 ? raw.x : (h == 1 ? raw.y : (h == 2 ? raw.z : raw.w)));
                                const v2f lo = __builtin_amdgcn_cvt_pk_f32_fp8(word, false);
                                const v2f hi = __builtin_amdgcn_cvt_pk_f32_fp8(word, true);
                                wv = make_float4(lo[0], lo[1], hi[0], hi[1]);
                            } else {
                                wv = raw;
                            }
#pragma unroll
                            for (int rg = 0; rg < RG; ++rg) {
                                acc[rg] = __builtin_amdgcn_mfma_f32_4x4x1f32(xa[rg].x, wv.x, acc[rg], 0, 0, 0);
                                acc[rg] = __builtin_amdgcn_mfma_f32_4x4x1f32(xa[rg].y, wv.y, acc[rg], 0, 0, 0);
                                acc[rg] = __builtin_amdgcn_mfma_f32_4x4x1f32(xa[rg].z, wv.z, acc[rg], 0, 0, 0);
                                acc[rg] = __builtin_amdgcn_mfma_f32_4x4x1f32(xa[rg].w, wv.w, acc[rg], 0, 0, 0);
                            }
#pragma unroll
                            for (int rg = 0; rg < RG; ++rg) xa[rg] = xb[rg];
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                    if (i + kAhead * kStepUnroll < left) {
#pragma unroll
                        for (int u = 0; u < kStepUnroll; ++u)
                            ws.q[a][u] = ws.base[ws.lane_off + (i + kAhead * kStepUnroll + u) * 64];
                    }
                }
            }
        }
        // when the partial sums reuse the memory of x, wait until every wave has read x
        if (red_aliases_x) __syncthreads();
        if (live) {
#pragma unroll
            for (int rg = 0; rg < RG; ++rg) {
                float4 o = make_float4(acc[rg][0], acc[rg][1], acc[rg][2], acc[rg][3]);
                *reinterpret_cast<float4 *>(red + task * red_task_stride(RG) + (rg * 4 + r4) * 4) = o;
            }
        }
        // next pass: same blocks, next kBlocksPerWg tasks
        ws.task = task + kBlocksPerWg;
        ws.base += sd.nsteps * 64;
        left -= sd.nsteps;
        // The batch that holds the next pass's first step becomes batch 0: a batch holds the
        // steps it was refilled with kAhead batches earlier, so after a pass of nsteps / 4
        // batches the roles have moved on by that count modulo kAhead.
        if (slot + 1 < sd.slots) {
            const int rot = (sd.nsteps / kStepUnroll) % kAhead;
#pragma unroll
            for (int u = 0; u < kStepUnroll; ++u) {
                float4 t_[kAhead];
#pragma unroll
                for (int i = 0; i < kAhead; ++i) t_[i] = ws.q[i][u];
                // constant indices on every path: the batches stay in registers
#pragma unroll
                for (int r = 1; r < kAhead; ++r)
                    if (rot == r) {
#pragma unroll
                        for (int i = 0; i < kAhead; ++i) ws.q[i][u] = t_[(i + r) % kAhead];
                    }
            }
        }
    }
}

// Sums of the K-slice partials of (group g, row) for its four columns, slices
// added in ascending order.  The loop is unrolled so the LDS reads overlap.
template <int RG>
__device__ __forceinline__ void reduce_tasks4(const float *red, int nks, int g, int row, float (&a)[4])
{
    const float *src = red + g * nks * red_task_stride(RG) + (row >> 2) * 16 + (row & 3);
    a[0] = a[1] = a[2] = a[3] = 0.f;
#pragma unroll 4
    for (int ks = 0; ks < nks; ++ks) {
        const float *q = src + ks * red_task_stride(RG);
        a[0] += q[0]; a[1] += q[4]; a[2] += q[8]; a[3] += q[12];
    }
}

__device__ __forceinline__ float sigmoidf_(float v) { return 1.0f / (1.0f + expf(-v)); }

struct Lds {
    float *xz, *red, *c, *part, *q, *hc;
    float *tail;                      // this rank's tail column: weight row, then [waves][kMaxSamples] partial sums
    float *b_pred, *b_out, *b_lstm;   // this rank's slices of the bias vectors
    // this rank's slices of the weight scales (e4m3 and e2m1 storage), indexed like a stage's
    // groups, [row][scale block of the stage's padded K]: rows of s_hh are (layer * units + u) * 4
    // + gate, s_ih likewise (a layer's table starts at layer * units * 4 * sc_nb_in), s_pred and
    // s_out by column
    unsigned char *s_pred, *s_out, *s_hh, *s_ih;   // exponent bytes of the power-of-two scales
};

// c state of this rank's units: [layer][sel][unit][row]
__device__ __forceinline__ float *c_slot(const DecodeParams &p, const Lds &l, int layer, int sel,
                                         int u, int row)
{
    return l.c + ((layer * 2 + sel) * p.nu_max + u) * p.rcap + row;
}
__device__ __forceinline__ float *h_slot(const DecodeParams &p, int team, int sel, int layer,
                                         int row)
{
    return p.hbuf + ((((long long)team * 2 + sel) * p.L + layer) * kMaxRows + row) * p.H;
}

// Fill RG*4 activation rows of `len` floats each into LDS from a global exchange
// buffer; the tail up to kpad and the rows beyond R are zero.  Loads are issued
// in batches so that their latencies overlap.
template <int WT>
__device__ __forceinline__ void fill_rows(const DecodeParams &p, const Wg &w, float *dst,
                                          int rows_pad, int len, int kpad, int layer, bool candidate)
{
    constexpr int NB = 6;
    const int kp2 = kpad >> 1;               // kpad is a multiple of 4
    const int total = rows_pad * kp2;        // pairs of floats
    const bool pairs = (len & 1) == 0;       // rows start 8-byte aligned
    for (int base = w.tid; base < total; base += NB * kThreads) {
        float2 v[NB];
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int idx = base + u * kThreads;
            v[u] = make_float2(0.f, 0.f);
            if (idx < total) {
                const int r = idx / kp2, k = (idx - r * kp2) * 2;
                if (r < c.R && k < len) {
                    const int sel = candidate ? (c.sel[r] ^ 1) : c.sel[r];
                    const float *src = h_slot(p, w.team, sel, layer, r) + k;
                    if (pairs) {
                        const unsigned long long q =
                            xload64(reinterpret_cast<const unsigned long long *>(src));
                        v[u].x = __uint_as_float((unsigned)q);
                        v[u].y = __uint_as_float((unsigned)(q >> 32));
                    } else {
                        v[u].x = xload(src);
                        if (k + 1 < len) v[u].y = xload(src + 1);
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            const int idx = base + u * kThreads;
            if (idx < total) {
                const int r = idx / kp2, k = (idx - r * kp2) * 2;
                x_store2<WT>(dst + r * p.xstride, k, v[u]);
            }
        }
    }
}

__device__ __forceinline__ void lstm_point(float gi, float gf, float gg, float go, float c_old,
                                           float &c_new, float &h_new)
{
    const float i_ = sigmoidf_(gi), f_ = sigmoidf_(gf), g_ = tanhf(gg), o_ = sigmoidf_(go);
    c_new = f_ * c_old + i_ * g_;
    h_new = o_ * tanhf(c_new);
}

// value of the lane a DPP control pairs the caller with
template <int CTRL>
__device__ __forceinline__ float dpp_f32(float v)
{
    const int i = (int)__float_as_uint(v);
    return __uint_as_float((unsigned)__builtin_amdgcn_update_dpp(i, i, CTRL, 0xf, 0xf, false));
}

// ---- prediction step for teams of up to four utterances --------------------------------
// Same arithmetic as prediction_step below, with two changes in how the hidden vectors
// travel.  (1) Every work-group keeps a copy of all hidden vectors of the team's rows in its
// LDS (committed and candidate, per layer): it reads every candidate vector anyway, as the
// input of the next stage, so the recurrent stage of the next step reads nothing from memory.
// (2) The exchanged values carry their step number: a work-group writes its slice as 64-bit
// words (step tag, float bits) and the readers poll the words themselves until the tag is the
// current step's, so a stage needs no barrier and no second round trip for the data.  A word
// is rewritten once per step, and nobody can reach step n + 1's store of a word before every
// work-group has read step n's (the stores of a stage need the complete input of the stage
// before, which needs every work-group's stores of that stage, made after its reads of the
// step before); the reset kernel clears the words, so a tag left by an earlier call is never
// current.
template <int NW>
__device__ __forceinline__ bool poll_words(const DecodeParams &p, Sync &sy, const unsigned long long *const (&src)[NW],
                                           unsigned tag, unsigned long long (&v)[NW])
{
    unsigned spins = 0;
    bool ok = true;
#pragma unroll
    for (int i = 0; i < NW; ++i) v[i] = src[i] ? xload64(src[i]) : ((unsigned long long)tag << 32);
    for (;;) {
        bool all = true;
#pragma unroll
        for (int i = 0; i < NW; ++i) all = all && (unsigned)(v[i] >> 32) == tag;
        if (all) break;
        ++spins;
        if ((spins & 127u) == 0 &&
            __hip_atomic_load(p.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
            ok = false;
            break;
        }
        if (spins > p.spin_limit) {
            __hip_atomic_store(p.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            ok = false;
            break;
        }
        __builtin_amdgcn_s_sleep(1);
#pragma unroll
        for (int i = 0; i < NW; ++i)
            if ((unsigned)(v[i] >> 32) != tag) v[i] = xload64(src[i]);
    }
    sy.polls += spins;
    if (!ok) c.bar_ok = 0;
    return ok;
}

__device__ __forceinline__ unsigned long long tagged(float v, unsigned tag)
{
    return ((unsigned long long)tag << 32) | __float_as_uint(v);
}

// value of lane `Q` of the caller's quad (four adjacent lanes)
template <int Q>
__device__ __forceinline__ float quad_lane(float v) { return dpp_f32<Q * 0x55>(v); }

template <int WT>
__device__ __forceinline__ bool prediction_step_fast(const DecodeParams &p, const Wg &w_in, Sync &sy, const Lds &l)
{
    Wg w = w_in;
    w.tid = rederive(w_in.tid); w.lane = w.tid & 63;
    constexpr int RG = 1;
    constexpr int KI = 2;                       // 64-bit words per row a thread polls: H, J <= 1024
    const int u0 = range_lo(w.rank, p.team_size, p.H), nu = range_hi(w.rank, p.team_size, p.H) - u0;
    const int xs = p.xstride, R = c.R;
    sy.pepoch += 1;
    const unsigned tag = sy.pepoch;
    const int r4 = w.lane & 3;
    const int selr = r4 < R ? c.sel[r4] : 0;    // rows beyond R stay zero in either copy
    float *hc = l.hc;                           // [2 selectors][L][4 rows][xs]
    const long long lay_stride = 4 * xs;
    // Candidate hidden vectors of layer `lay`, all rows: wait for every word, keep them in LDS.
    auto receive_h = [&](int lay) -> bool {
        const unsigned long long *base = p.xh + (((long long)w.team * p.L + lay) * kMaxRows) * p.H;
        const unsigned long long *src[4 * KI];
        unsigned long long v[4 * KI];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < KI; ++i) {
                const int k = w.tid + i * kThreads;
                src[r * KI + i] = (r < R && k < p.H) ? base + (long long)r * p.H + k : nullptr;
            }
        if (!poll_words<4 * KI>(p, sy, src, tag, v)) return false;
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < KI; ++i) {
                const int k = w.tid + i * kThreads;
                if (r < R && k < p.H)
                    x_store<WT>(hc + (((c.sel[r] ^ 1) * p.L + lay) * 4 + r) * xs, k,
                                __uint_as_float((unsigned)v[r * KI + i]));
            }
        return true;
    };
    // LSTM cell of (layer, unit u, row r) on the four lanes of a quad: lane j holds the
    // pre-activation of gate j (input, forget, cell, output)
    auto cell = [&](int layer, int u, int r, int j, float pre) {
        const float act = j == 2 ? tanhf(pre) : sigmoidf_(pre);
        const float i_ = quad_lane<0>(act), f_ = quad_lane<1>(act), g_ = quad_lane<2>(act), o_ = quad_lane<3>(act);
        if (j == 0) {
            const float cn = f_ * *c_slot(p, l, layer, c.sel[r], u, r) + i_ * g_;
            const float hn = o_ * tanhf(cn);
            *c_slot(p, l, layer, c.sel[r] ^ 1, u, r) = cn;
            xstore64(p.xh + (((long long)w.team * p.L + layer) * kMaxRows + r) * p.H + u0 + u, tagged(hn, tag));
        }
    };
    PROF_MARK(w, 18);
    // the row of the folded embedding table this thread will add after stage 0 (layer 0 of its
    // first (unit, row, gate) element): requested now, used when the stage's sums are there
    float t0_first = 0.f;
    {
        const int e = w.tid >> 2, j = w.tid & 3;
        if (w.tid < p.L * nu * R * 4 && e < nu * R) {
            const int u = e / R, r = e - u * R;
            t0_first = p.T0[((long long)c.last[r] * p.H + (u0 + u)) * 4 + j];
        }
    }
    // stage 0: recurrent parts of every layer from the committed vectors in LDS
    WeightStream ws;
    stream_begin(ws, p.st0, w, w.rank, p.L * nu * p.st0.nks);
    PROF_MARK(w, 0);
    run_stage<RG, WT>(p.st0, w, p.L * nu * p.st0.nks, ws, hc + (long long)selr * p.L * lay_stride, xs,
                      (int)lay_stride, nu > 0 ? nu : 1, l.red, false, l.s_hh);
    const int ng_all_p = (p.J + 3) / 4;
    const int gp0 = range_lo(w.rank, p.team_size, ng_all_p);
    const int ngp = range_hi(w.rank, p.team_size, ng_all_p) - gp0;
    if (p.L > 1) stream_begin(ws, p.stl[1], w, w.rank, nu * p.stl[1].nks);
    else stream_begin(ws, p.spred, w, w.rank, ngp * p.spred.nks);
    __syncthreads();
    PROF_MARK(w, 1);
    for (int e4 = w.tid; e4 < p.L * nu * R * 4; e4 += kThreads) {
        const int e = e4 >> 2, j = e4 & 3;
        const int layer = e / (nu * R);
        const int rem = e - layer * nu * R;
        const int u = rem / R, r = rem - u * R;
        const float *src = l.red + (layer * nu + u) * p.st0.nks * red_task_stride(RG) + j * 4 + r;
        float a = 0.f;
        for (int ks = 0; ks < p.st0.nks; ++ks) a += src[ks * red_task_stride(RG)];
        if (layer == 0) {
            a += e4 == w.tid ? t0_first : p.T0[((long long)c.last[r] * p.H + (u0 + u)) * 4 + j];
            cell(0, u, r, j, a);
        } else {
            l.part[((layer * p.nu_max + u) * p.rcap + r) * 4 + j] = a + l.b_lstm[(layer * p.nu_max + u) * 4 + j];
        }
    }
    PROF_MARK(w, 2);
    // stages 1..L-1: input part of layer `layer` from the candidate h of the layer below
#pragma unroll
    for (int layer = 1; layer < kMaxLayers; ++layer) {
        if (layer >= p.L) break;
        const StageDev &sd = p.stl[layer];
        if (!receive_h(layer - 1)) return false;
        __syncthreads();
        PROF_MARK(w, 4);
        run_stage<RG, WT>(sd, w, nu * sd.nks, ws, hc + ((long long)(selr ^ 1) * p.L + (layer - 1)) * lay_stride, xs,
                          0, 1 << 30, l.red, false, l.s_ih + layer * nu * 4 * p.sc_nb_in);
        if (layer + 1 < kMaxLayers && layer + 1 < p.L)
            stream_begin(ws, p.stl[layer + 1 < kMaxLayers ? layer + 1 : layer], w, w.rank,
                         nu * p.stl[layer + 1 < kMaxLayers ? layer + 1 : layer].nks);
        else stream_begin(ws, p.spred, w, w.rank, ngp * p.spred.nks);
        __syncthreads();
        PROF_MARK(w, 5);
        for (int e4 = w.tid; e4 < nu * R * 4; e4 += kThreads) {
            const int e = e4 >> 2, j = e4 & 3;
            const int u = e / R, r = e - u * R;
            const float *src = l.red + u * sd.nks * red_task_stride(RG) + j * 4 + r;
            float a = 0.f;
            for (int ks = 0; ks < sd.nks; ++ks) a += src[ks * red_task_stride(RG)];
            a += l.part[((layer * p.nu_max + u) * p.rcap + r) * 4 + j];
            cell(layer, u, r, j, a);
        }
        PROF_MARK(w, 6);
    }
    // prediction-side joint projection
    if (!receive_h(p.L - 1)) return false;
    __syncthreads();
    PROF_MARK(w, 8);
    run_stage<RG, WT>(p.spred, w, ngp * p.spred.nks, ws, hc + ((long long)(selr ^ 1) * p.L + (p.L - 1)) * lay_stride,
                      xs, 0, 1 << 30, l.red, false, l.s_pred);
    __syncthreads();
    PROF_MARK(w, 9);
    for (int e4 = w.tid; e4 < ngp * R * 4; e4 += kThreads) {
        const int e = e4 >> 2, j = e4 & 3;
        const int g = e / R, r = e - g * R;
        const float *src = l.red + g * p.spred.nks * red_task_stride(RG) + j * 4 + r;
        float a = 0.f;
        for (int ks = 0; ks < p.spred.nks; ++ks) a += src[ks * red_task_stride(RG)];
        const int col = (gp0 + g) * 4 + j;
        if (col < p.J)
            xstore64(p.xq + ((long long)w.team * kMaxRows + r) * p.J + col, tagged(a + l.b_pred[g * 4 + j], tag));
    }
    PROF_MARK(w, 10);
    {
        // q of the rows this joint group searches for
        const unsigned long long *src[4 * KI];
        unsigned long long v[4 * KI];
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
#pragma unroll
            for (int i = 0; i < KI; ++i) {
                const int r = w.jg + i4 * p.groups, k = w.tid + i * kThreads;
                src[i4 * KI + i] = (r < R && k < p.J) ? p.xq + ((long long)w.team * kMaxRows + r) * p.J + k : nullptr;
            }
        if (!poll_words<4 * KI>(p, sy, src, tag, v)) return false;
#pragma unroll
        for (int i4 = 0; i4 < 4; ++i4)
#pragma unroll
            for (int i = 0; i < KI; ++i) {
                const int r = w.jg + i4 * p.groups, k = w.tid + i * kThreads;
                if (r < R && k < p.J) l.q[i4 * p.qstride + k] = __uint_as_float((unsigned)v[i4 * KI + i]);
            }
    }
    __syncthreads();
    PROF_MARK(w, 12);
    return c.bar_ok != 0;
}

// One prediction-network step for all rows of the team, from (last, committed
// state) to the candidate state and q = W_pred h'_top + b_pred.
template <int RG, int WT>
__device__ __forceinline__ bool prediction_step(const DecodeParams &p, const Wg &w, Sync &sy, const Lds &l)
{
    if constexpr (RG == 1) {
        if (p.fast_pred) return prediction_step_fast<WT>(p, w, sy, l);
    }
    const int u0 = range_lo(w.rank, p.team_size, p.H), nu = range_hi(w.rank, p.team_size, p.H) - u0;
    const int rows_pad = RG * 4;
    const int inp_stride = rows_pad * p.xstride;
    // stage 0: recurrent parts of every layer, layer 0 completes
    PROF_MARK(w, 18);
    WeightStream ws;
    stream_begin(ws, p.st0, w, w.rank, p.L * nu * p.st0.nks);
    for (int layer = 0; layer < p.L; ++layer)
        fill_rows<WT>(p, w, l.xz + layer * inp_stride, rows_pad, p.H, p.st0.kpad, layer, false);
    __syncthreads();
    // the additive term of this thread's first epilogue item (embedding term of layer 0,
    // bias of the layers above) is fetched before the product so its latency is hidden
    PROF_MARK(w, 0);
    float4 pre = make_float4(0.f, 0.f, 0.f, 0.f);
    if (w.tid < p.L * nu * c.R) {
        const int layer = w.tid / (nu * c.R);
        const int rem = w.tid - layer * nu * c.R;
        const int u = rem / c.R, r = rem - u * c.R;
        if (layer == 0)
            pre = *reinterpret_cast<const float4 *>(p.T0 + ((long long)c.last[r] * p.H + (u0 + u)) * 4);
    }
    run_stage<RG, WT>(p.st0, w, p.L * nu * p.st0.nks, ws, l.xz, p.xstride, inp_stride, nu > 0 ? nu : 1,
                  l.red, false, l.s_hh);
    // the next stage's weights start moving while this one finishes and the team meets
    const int ng_all_p = (p.J + 3) / 4;
    const int gp0 = range_lo(w.rank, p.team_size, ng_all_p);
    const int ngp = range_hi(w.rank, p.team_size, ng_all_p) - gp0;
    if (p.L > 1) stream_begin(ws, p.stl[1], w, w.rank, nu * p.stl[1].nks);
    else stream_begin(ws, p.spred, w, w.rank, ngp * p.spred.nks);
    __syncthreads();
    PROF_MARK(w, 1);
    for (int e = w.tid; e < p.L * nu * c.R; e += kThreads) {
        const int layer = e / (nu * c.R);
        const int rem = e - layer * nu * c.R;
        const int u = rem / c.R, r = rem - u * c.R;
        const int g = layer * nu + u;
        float a[4];
        reduce_tasks4<RG>(l.red, p.st0.nks, g, r, a);
        if (layer == 0) {
            // (an assignment under a condition, not a conditional expression on the two objects:
            // that would make the compiler address both through one generic pointer, one of
            // them on the stack)
            float4 t0 = pre;
            if (e != w.tid)
                t0 = *reinterpret_cast<const float4 *>(p.T0 + ((long long)c.last[r] * p.H + (u0 + u)) * 4);
            float cn, hn;
            lstm_point(a[0] + t0.x, a[1] + t0.y, a[2] + t0.z, a[3] + t0.w,
                       *c_slot(p, l, 0, c.sel[r], u, r), cn, hn);
            *c_slot(p, l, 0, c.sel[r] ^ 1, u, r) = cn;
            xstore(h_slot(p, w.team, c.sel[r] ^ 1, 0, r) + u0 + u, hn);
        } else {
            const float4 bl = *reinterpret_cast<const float4 *>(l.b_lstm + (layer * p.nu_max + u) * 4);
            float *dst = l.part + ((layer * p.nu_max + u) * p.rcap + r) * 4;
            dst[0] = a[0] + bl.x; dst[1] = a[1] + bl.y; dst[2] = a[2] + bl.z; dst[3] = a[3] + bl.w;
        }
    }
    PROF_MARK(w, 2);
    if (!team_barrier(p, w, sy)) return false;
    PROF_MARK(w, 3);
    // stages 1..L-1: input part of layer `layer` from the candidate h of the layer below
#pragma unroll
    for (int layer = 1; layer < kMaxLayers; ++layer) {
        if (layer >= p.L) break;
        const StageDev &sd = p.stl[layer];
        fill_rows<WT>(p, w, l.xz, rows_pad, p.H, sd.kpad, layer - 1, true);
        __syncthreads();
        PROF_MARK(w, 4);
        run_stage<RG, WT>(sd, w, nu * sd.nks, ws, l.xz, p.xstride, 0, 1 << 30, l.red, false, l.s_ih + layer * nu * 4 * p.sc_nb_in);
        if (layer + 1 < kMaxLayers && layer + 1 < p.L)
            stream_begin(ws, p.stl[layer + 1 < kMaxLayers ? layer + 1 : layer], w, w.rank,
                         nu * p.stl[layer + 1 < kMaxLayers ? layer + 1 : layer].nks);
        else stream_begin(ws, p.spred, w, w.rank, ngp * p.spred.nks);
        __syncthreads();
        PROF_MARK(w, 5);
        for (int e = w.tid; e < nu * c.R; e += kThreads) {
            const int u = e / c.R, r = e - u * c.R;
            float a[4];
            reduce_tasks4<RG>(l.red, sd.nks, u, r, a);
            const float *pt = l.part + ((layer * p.nu_max + u) * p.rcap + r) * 4;
            float cn, hn;
            lstm_point(a[0] + pt[0], a[1] + pt[1], a[2] + pt[2], a[3] + pt[3],
                       *c_slot(p, l, layer, c.sel[r], u, r), cn, hn);
            *c_slot(p, l, layer, c.sel[r] ^ 1, u, r) = cn;
            xstore(h_slot(p, w.team, c.sel[r] ^ 1, layer, r) + u0 + u, hn);
        }
        PROF_MARK(w, 6);
        if (!team_barrier(p, w, sy)) return false;
        PROF_MARK(w, 7);
    }
    // prediction-side joint projection
    {
        const int g0 = gp0, ng = ngp;
        fill_rows<WT>(p, w, l.xz, rows_pad, p.H, p.spred.kpad, p.L - 1, true);
        __syncthreads();
        PROF_MARK(w, 8);
        run_stage<RG, WT>(p.spred, w, ng * p.spred.nks, ws, l.xz, p.xstride, 0, 1 << 30, l.red, false, l.s_pred);
        __syncthreads();
        PROF_MARK(w, 9);
        for (int e = w.tid; e < ng * c.R; e += kThreads) {
            const int g = e / c.R, r = e - g * c.R;
            float a[4];
            reduce_tasks4<RG>(l.red, p.spred.nks, g, r, a);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = (g0 + g) * 4 + j;
                if (col < p.J)
                    xstore(p.qbuf + ((long long)w.team * kMaxRows + r) * p.J + col, a[j] + l.b_pred[g * 4 + j]);
            }
        }
        PROF_MARK(w, 10);
        if (!team_barrier(p, w, sy)) return false;
        PROF_MARK(w, 11);
        if (p.q_in_lds) {
            // q of the rows this joint group searches for, read once per prediction step
            constexpr int NB = 6;
            const int own = c.R > w.jg ? (c.R - w.jg + p.groups - 1) / p.groups : 0;
            const int total = own * p.qstride;
            for (int base = w.tid; base < total; base += NB * kThreads) {
                float v[NB];
#pragma unroll
                for (int u = 0; u < NB; ++u) {
                    const int idx = base + u * kThreads;
                    v[u] = 0.f;
                    if (idx < total) {
                        const int j = idx / p.qstride, k = idx - j * p.qstride;
                        const int r = w.jg + j * p.groups;
                        if (k < p.J)
                            v[u] = xload(p.qbuf + ((long long)w.team * kMaxRows + r) * p.J + k);
                    }
                }
#pragma unroll
                for (int u = 0; u < NB; ++u) {
                    const int idx = base + u * kThreads;
                    if (idx < total) l.q[idx] = v[u];
                }
            }
            __syncthreads();
        }
        PROF_MARK(w, 12);
    }
    return true;
}

// ---- argmax candidates as 64-bit keys -------------------------------------------------
// A candidate (logit v, column idx) is packed so that an unsigned comparison orders by value
// first and, among equal values, by the lower column: high word = the float's bits mapped to
// an order-preserving unsigned (-0 is made +0 first), low 16 bits = 0xffff - idx.  Bits 16-31
// carry the step tag while a key travels between work-groups and are zero otherwise.  Logits
// have to be finite (a NaN would order above every number).
__device__ __forceinline__ unsigned long long make_key(float v, int idx)
{
    const unsigned u = __float_as_uint(v + 0.0f);
    const unsigned o = u ^ ((unsigned)((int)u >> 31) | 0x80000000u);
    return ((unsigned long long)o << 32) | (unsigned)(0xffff - idx);
}
__device__ __forceinline__ float key_value(unsigned long long k)
{
    const unsigned o = (unsigned)(k >> 32);
    return __uint_as_float(o ^ ((o >> 31) ? 0x80000000u : 0xffffffffu));
}
__device__ __forceinline__ int key_index(unsigned long long k) { return 0xffff - (int)(k & 0xffffu); }

// max of the keys of a lane and of the lane a DPP control pairs it with
// (0xB1: lane ^ 1, 0x4E: lane ^ 2, 0x141: mirror within 8 lanes, 0x140: mirror within 16)
template <int CTRL>
__device__ __forceinline__ unsigned long long key_max_dpp(unsigned long long k)
{
    const int lo = (int)(unsigned)k, hi = (int)(unsigned)(k >> 32);
    const int olo = __builtin_amdgcn_update_dpp(lo, lo, CTRL, 0xf, 0xf, false);
    const int ohi = __builtin_amdgcn_update_dpp(hi, hi, CTRL, 0xf, 0xf, false);
    const unsigned long long o = ((unsigned long long)(unsigned)ohi << 32) | (unsigned)olo;
    return o > k ? o : k;
}
// max over groups of 8 (all 8 lanes get it) or 16 adjacent lanes
__device__ __forceinline__ unsigned long long key_max8(unsigned long long k)
{
    k = key_max_dpp<0xB1>(k); k = key_max_dpp<0x4E>(k); return key_max_dpp<0x141>(k);
}
__device__ __forceinline__ unsigned long long key_max16(unsigned long long k)
{
    return key_max_dpp<0x140>(key_max8(k));
}
// log-sum-exp pairs (maximum m, sum s of exp(x - m)) combined the same way
__device__ __forceinline__ void lse_merge(float &m, float &s, float om, float os)
{
    if (om > m) { s = s * expf(m - om) + os; m = om; }
    else if (om > -INFINITY) s += os * expf(om - m);
}
template <int CTRL>
__device__ __forceinline__ void lse_merge_dpp(float &m, float &s)
{
    const float om = dpp_f32<CTRL>(m), os = dpp_f32<CTRL>(s);
    lse_merge(m, s, om, os);
}

// An argmax partial as exchanged between the ranks of a joint group: a key with the 16-bit tag
// (the joint step it belongs to, modulo 65536) in bits 16-31.  Readers poll a slot until
// its tag is the current step's, so the exchange needs no separate barrier.  Why a stale tag
// can never equal the current one, however many joint steps a call takes: the slots of a step
// are chosen by the parity of the step number, every rank rewrites all slots s < ns of that
// parity at every such step (valid sample or not), readers read only slots s < ns, and ns never
// grows during a call (label looping keeps it constant, Algorithm 1 shrinks it on the last
// frames only).  So what a reader can find in a slot is the current step's word or the one
// written two steps earlier, whose tag differs by 2 modulo 65536; the value 0 the reset kernel
// leaves is only ever found before step 1 or 2 has been written, and those tags are 1 and 2.
__device__ __forceinline__ unsigned long long with_tag(unsigned long long key, unsigned tag)
{
    return key | ((unsigned long long)(tag & 0xffffu) << 16);
}
__device__ __forceinline__ bool has_tag(unsigned long long word, unsigned tag)
{
    return (unsigned)((word >> 16) & 0xffffu) == (tag & 0xffffu);
}

// Read up to four tagged words (slots base[r0], base[r0 + stride], ...; n of them) with all
// loads in flight together, polling again only for those that are not there yet.  Bounded:
// gives up (and raises the abort flag) after spin_limit polls or when another work-group has
// raised it.  Tags are stripped from what is returned.  With PRELOADED the caller has already
// issued the first round of loads into `out` (read_words4), together with those of another set
// of words it waits for first.
__device__ __forceinline__ void read_words4(const unsigned long long *base, int stride, int n,
                                            unsigned long long (&out)[4])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) out[i] = i < n ? xload64(base + i * stride) : 0ull;
}
template <bool PRELOADED = false>
__device__ __forceinline__ void wait_words4(const DecodeParams &p, Sync &sy, const unsigned long long *base,
                                            int stride, int n, unsigned tag, unsigned long long (&out)[4])
{
    unsigned spins = 0;
    if (!PRELOADED) read_words4(base, stride, n, out);
    for (;;) {
        bool all = true;
#pragma unroll
        for (int i = 0; i < 4; ++i) all = all && (i >= n || has_tag(out[i], tag));
        if (all) break;
        ++spins;
        if ((spins & 127u) == 0 &&
            __hip_atomic_load(p.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
            c.bar_ok = 0;
            break;
        }
        if (spins > p.spin_limit) {
            __hip_atomic_store(p.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            c.bar_ok = 0;
            break;
        }
        __builtin_amdgcn_s_sleep(1);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (i < n && !has_tag(out[i], tag)) out[i] = xload64(base + i * stride);
    }
    sy.polls += spins;
#pragma unroll
    for (int i = 0; i < 4; ++i) out[i] &= ~0xffff0000ull;
}

// Joint network + argmax for the c.ns samples listed in c.s_row / c.s_frame /
// c.s_valid.  Leaves c.s_k, c.s_v (token argmax and its logit) and c.s_d
// (duration index) for every valid sample.
template <int RG, int WT>
__device__ __forceinline__ bool joint_step(const DecodeParams &p, const Wg &w_in, Sync &sy, const Lds &l)
{
    Wg w = w_in;
    w.tid = rederive(w_in.tid); w.lane = w.tid & 63;
    const int ns = c.ns;
    const int rows_pad = RG * 4;
    const int kpad = p.sjoint.kpad;
    sy.jepoch += 1;
    const unsigned tag = sy.jepoch;
    const int parity = (int)(tag & 1u);
    const int ng_all = (p.nout_m + 3) / 4;
    const int g0 = range_lo(w.jrank, p.jteam_size, ng_all);
    const int ng = range_hi(w.jrank, p.jteam_size, ng_all) - g0;
    // a rank with a tail column has one more candidate per sample than it has output groups
    const bool has_tail = w.jrank < p.n_tail;
    const int ngx = ng + (has_tail ? 1 : 0);
    PROF_MARK(w, 18);
    // z = relu(P[b, frame] + q[row]) for every sample.  Wave v builds the samples v, v + 8, ...,
    // so a sample's row addresses are uniform over the wave; a lane takes four floats at k = 4 *
    // (lane, lane + 64, lane + 128).  The loads of the projected frames go out first, then the
    // first batches of the weight stream (a wave's loads return in order and z is needed
    // first), then z is formed and written to LDS.
    WeightStream ws;
    {
        const int k4n = kpad >> 2;                 // float4 per z row, zero padding included
        const int j4 = p.J >> 2;                   // float4 of a row (J is a multiple of 4)
        constexpr int SPW = (RG * 4 + kWaves - 1) / kWaves;    // samples per wave
        float4 pe[SPW][3];
        int valid[SPW], qoff[SPW];
#pragma unroll
        for (int i = 0; i < SPW; ++i) {
            const int s = w.wave + i * kWaves;
            valid[i] = 0; qoff[i] = 0;
#pragma unroll
            for (int u = 0; u < 3; ++u) pe[i][u] = make_float4(0.f, 0.f, 0.f, 0.f);
            // (both were worked out when the samples were set up: two independent reads here)
            const int pidx = s < ns ? __builtin_amdgcn_readfirstlane(c.s_pidx[s]) : -1;
            const int qo = __builtin_amdgcn_readfirstlane(c.s_qoff[s & (kMaxSamples - 1)]);
            valid[i] = pidx >= 0;
            if (valid[i]) {
                qoff[i] = qo;
                const float *pr = p.P + (long long)pidx * p.J;
#pragma unroll
                for (int u = 0; u < 3; ++u) {
                    const int k4 = w.lane + 64 * u;
                    if (64 * u < j4)       // uniform; lanes past the row read its first float4
                        pe[i][u] = reinterpret_cast<const float4 *>(pr)[k4 < j4 ? k4 : 0];
                }
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        stream_begin(ws, p.sjoint, w, w.jrank, ng * p.sjoint.nks);
        __builtin_amdgcn_sched_barrier(0);
        PROF_MARK(w, 22);
#pragma unroll
        for (int i = 0; i < SPW; ++i) {
            const int s = w.wave + i * kWaves;
            if (s >= rows_pad) break;
            float *zrow = l.xz + s * p.xstride;
#pragma unroll
            for (int u = 0; u < 3; ++u) {
                const int k4 = w.lane + 64 * u;
                if (k4 >= k4n) break;
                const int k = k4 * 4;
                float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
                if (valid[i] && k < p.J) {
                    float4 qv;
                    if (p.q_in_lds) {
                        qv = *reinterpret_cast<const float4 *>(l.q + qoff[i] + k);
                    } else {
                        const float *qr = p.qbuf + ((long long)w.team * kMaxRows + qoff[i]) * p.J + k;
                        qv = make_float4(xload(qr), xload(qr + 1), xload(qr + 2), xload(qr + 3));
                    }
                    z = make_float4(fmaxf(pe[i][u].x + qv.x, 0.f), fmaxf(pe[i][u].y + qv.y, 0.f),
                                    fmaxf(pe[i][u].z + qv.z, 0.f), fmaxf(pe[i][u].w + qv.w, 0.f));
                }
                x_store4<WT>(zrow, k, z);
            }
            // joint layers wider than 768: the rest of the row, loaded where it is used
            for (int k4 = w.lane + 192; k4 < k4n; k4 += 64) {
                const int k = k4 * 4;
                float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
                if (valid[i] && k < p.J) {
                    const int sidx = w.wave + i * kWaves;
                    const int r = c.s_row[sidx];
                    const float *pr = p.P + ((long long)c.b[r] * p.T + c.s_frame[sidx]) * p.J + k;
                    const float *qr = p.qbuf + ((long long)w.team * kMaxRows + r) * p.J + k;
                    float pv[4], qv[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        pv[j] = pr[j];
                        qv[j] = p.q_in_lds ? l.q[qoff[i] + k + j] : xload(qr + j);
                    }
                    z = make_float4(fmaxf(pv[0] + qv[0], 0.f), fmaxf(pv[1] + qv[1], 0.f),
                                    fmaxf(pv[2] + qv[2], 0.f), fmaxf(pv[3] + qv[3], 0.f));
                }
                x_store4<WT>(zrow, k, z);
            }
        }
        PROF_MARK(w, 23);
    }
    __syncthreads();
    PROF_MARK(w, 13);
    if (has_tail) {
        // This rank's tail column (output column nout_m + jrank) for every sample, while the
        // first weight batches of the stage are on their way: wave v takes the v-th eighth of
        // K, 64 / rows_pad adjacent lanes share a sample, and the per-wave sums go to LDS.
        constexpr int NSUB = 64 / (RG * 4);
        const int k4n = (p.J + 3) >> 2, kw4 = (k4n + kWaves - 1) / kWaves;
        const int s = w.lane / NSUB, sub = w.lane % NSUB;
        const int lo = w.wave * kw4, hi = min(lo + kw4, k4n);
        const float *zrow = l.xz + s * p.xstride;
        float acc = 0.f;
        for (int k4 = lo + sub; k4 < hi; k4 += NSUB) {
            const float4 z = x_load4<WT>(zrow, k4 * 4);
            const float4 wv = *reinterpret_cast<const float4 *>(l.tail + k4 * 4);
            acc = fmaf(z.x, wv.x, acc); acc = fmaf(z.y, wv.y, acc);
            acc = fmaf(z.z, wv.z, acc); acc = fmaf(z.w, wv.w, acc);
        }
        if (NSUB >= 2) acc += dpp_f32<0xB1>(acc);
        if (NSUB >= 4) acc += dpp_f32<0x4E>(acc);
        if (NSUB >= 8) acc += dpp_f32<0x141>(acc);
        if (NSUB >= 16) acc += dpp_f32<0x140>(acc);
        if (sub == 0) l.tail[((p.J + 3) & ~3) + w.wave * kMaxSamples + s] = acc;
    }
    // with one slot the partial sums may overwrite z once every wave is done with it; the
    // output bias goes into the accumulators of every group's first K slice
    const bool alias = p.sjoint.slots == 1;
    float *red = alias ? l.xz : l.red;
    run_stage<RG, WT>(p.sjoint, w, ng * p.sjoint.nks, ws, l.xz, p.xstride, 0, 1 << 30, red, alias, l.s_out, l.b_out);
    __syncthreads();
    PROF_MARK(w, 14);
    // Per sample, this rank's best token column and best duration column, in two steps through
    // LDS.  First one thread per (sample, group of four columns): the K-slice partials are
    // added and the best of the four columns becomes a key.  The keys go where nothing is
    // live: into the partial-sum region when the sums sit in the z rows, else into the z rows.
    unsigned long long *cand = reinterpret_cast<unsigned long long *>(alias ? l.red : l.xz);
    unsigned long long *cand_d = cand + ns * ngx;
    // for the scores: per (sample, group) the sum of exp(logit - the group's maximum) over its
    // token columns, merged below like the keys (asked for only when the caller wants scores)
    float *se_part = reinterpret_cast<float *>(cand + 2 * ns * ngx) + kMaxSamples;   // [ns][ngx]
    float *tail_sum = l.tail + ((p.J + 3) & ~3);
    {
        int nsp = 1, lg = 0;
        while (nsp < ns) { nsp <<= 1; ++lg; }
        const int s = w.tid & (nsp - 1);
        for (int g = w.tid >> lg; g < ng; g += kThreads >> lg) {
            if (s >= ns) continue;
            float a[4];
            reduce_tasks4<RG>(red, p.sjoint.nks, g, s, a);
            unsigned long long kt = 0ull, kd = 0ull;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int col = (g0 + g) * 4 + j;
                if (col < p.VT) { const unsigned long long k = make_key(a[j], col); kt = k > kt ? k : kt; }
                else if (col < p.NOUT) { const unsigned long long k = make_key(a[j], col - p.VT); kd = k > kd ? k : kd; }
            }
            cand[s * ngx + g] = kt;
            if (p.D > 0) cand_d[s * ngx + g] = kd;
            if (p.logps) {
                float m4 = -INFINITY, se = 0.f;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if ((g0 + g) * 4 + j < p.VT) m4 = fmaxf(m4, a[j]);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    if ((g0 + g) * 4 + j < p.VT) se += expf(a[j] - m4);
                se_part[s * ngx + g] = se;
            }
        }
        if (has_tail && w.tid < ns) {
            // the tail column's logit: its bias plus the waves' sums; kept in the first wave's
            // slot for the scores
            float a = p.b_out[p.nout_m + w.jrank];
#pragma unroll
            for (int v = 0; v < kWaves; ++v) a += tail_sum[v * kMaxSamples + w.tid];
            tail_sum[w.tid] = a;
            const int col = p.nout_m + w.jrank;
            cand[w.tid * ngx + ng] = col < p.VT ? make_key(a, col) : 0ull;
            if (p.D > 0) cand_d[w.tid * ngx + ng] = col < p.VT ? 0ull : make_key(a, col - p.VT);
            if (p.logps) se_part[w.tid * ngx + ng] = col < p.VT ? 1.f : 0.f;
        }
    }
    __syncthreads();
    PROF_MARK(w, 20);
    // then eight adjacent lanes per sample scan the groups and publish the rank's partial
    if (w.wave * 8 < ns) {
        const int s = w.tid >> 3, sub = w.tid & 7;
        unsigned long long kt = 0ull, kd = 0ull;
        float lm = -INFINITY, ls = 0.f;        // running (maximum, sum of exp relative to it)
        if (s < ns)
            for (int g = sub; g < ngx; g += 8) {
                const unsigned long long k = cand[s * ngx + g];
                kt = k > kt ? k : kt;
                if (p.D > 0) { const unsigned long long d = cand_d[s * ngx + g]; kd = d > kd ? d : kd; }
                if (p.logps && k) lse_merge(lm, ls, key_value(k), se_part[s * ngx + g]);
            }
        kt = key_max8(kt);
        if (p.D > 0) kd = key_max8(kd);
        if (p.logps) { lse_merge_dpp<0xB1>(lm, ls); lse_merge_dpp<0x4E>(lm, ls); lse_merge_dpp<0x141>(lm, ls); }
        if (s < ns && sub == 0) {
            const long long o =
                (((long long)(w.team * p.groups + w.jg) * 2 + parity) * kMaxSamples + s) * p.jteam_size + w.jrank;
            xstore64(p.part + o, with_tag(kt, tag));
            if (p.D > 0) xstore64(p.dpart + o, with_tag(kd, tag));
            // the rank's sum, relative to its own maximum (the value of kt), travels as a float
            // in the high word (it is positive: no key order needed)
            if (p.logps) xstore64(p.lpart + o, with_tag((unsigned long long)__float_as_uint(ls) << 32, tag));
        }
    }
    PROF_MARK(w, 15);
    // final argmax over the ranks: sixteen adjacent lanes per sample, each with up to four
    // ranks' partials in flight at a time
    if (w.wave * 4 < ns) {
        const int s = w.tid >> 4, sub = w.tid & 15;
        const bool mine = s < ns && c.s_valid[s];
        unsigned long long kt = 0ull, kd = 0ull;
        float lm = -INFINITY, ls = 0.f;
        if (mine) {
            const long long o =
                (((long long)(w.team * p.groups + w.jg) * 2 + parity) * kMaxSamples + s) * p.jteam_size;
            for (int r0 = sub; r0 < p.jteam_size; r0 += 64) {
                const int n = min(4, (p.jteam_size - r0 + 15) >> 4);
                unsigned long long wd[4], wdur[4];
                unsigned long long wl[4];
                if (p.D > 0) read_words4(p.dpart + o + r0, 16, n, wdur);   // in flight with the token words
                if (p.logps) read_words4(p.lpart + o + r0, 16, n, wl);
                wait_words4(p, sy, p.part + o + r0, 16, n, tag, wd);
                if (p.logps) {
                    wait_words4<true>(p, sy, p.lpart + o + r0, 16, n, tag, wl);
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (i < n && wd[i]) lse_merge(lm, ls, key_value(wd[i]), __uint_as_float((unsigned)(wl[i] >> 32)));
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) kt = wd[i] > kt ? wd[i] : kt;
                if (p.D > 0) {
                    wait_words4<true>(p, sy, p.dpart + o + r0, 16, n, tag, wdur);
#pragma unroll
                    for (int i = 0; i < 4; ++i) kd = wdur[i] > kd ? wdur[i] : kd;
                }
            }
        }
        kt = key_max16(kt);
        if (p.D > 0) kd = key_max16(kd);
        if (p.logps) {
            lse_merge_dpp<0xB1>(lm, ls); lse_merge_dpp<0x4E>(lm, ls);
            lse_merge_dpp<0x141>(lm, ls); lse_merge_dpp<0x140>(lm, ls);
        }
        if (mine && sub == 0) {
            // no candidate at all cannot happen (every rank owns at least one token column or
            // publishes key 0, and rank 0 always owns column 0); keep the index in range anyway
            int bi = kt ? key_index(kt) : p.blank;
            if ((unsigned)bi >= (unsigned)p.VT) bi = p.blank;
            const int di = (p.D > 0 && kd) ? key_index(kd) : 0;
            c.s_k[s] = bi; c.s_v[s] = key_value(kt); c.s_d[s] = di < p.D ? di : 0;
            c.s_lp[s] = p.logps ? -logf(ls) : 0.f;      // the maximum is its own reference: logit - lm = 0
        }
    }
    __syncthreads();
    PROF_MARK(w, 17);
    return c.bar_ok != 0;
}

// Row r emits label k at frame t (rank 0 writes the outputs).
__device__ __forceinline__ void emit_row(const DecodeParams &p, const Wg &w, int r, int k,
                                         int t, float v, float lp, int dval)
{
    const int n = c.cnt[r];
    if (w.jrank == 0) {
        if (n < p.cap) {
            const long long o = (long long)c.b[r] * p.cap + n;
            p.tokens[o] = k;
            if (p.frames) p.frames[o] = t;
            if (p.logits) p.logits[o] = v;
            if (p.logps) p.logps[o] = lp;
            if (p.durs) p.durs[o] = dval;
        } else {
            c.st_overflow = 1;
        }
    }
    c.cnt[r] = n + 1;
    c.last[r] = k;
    c.sel[r] ^= 1;     // the candidate state becomes the state
}

// Row r has its last label: publish its count and, when the caller asked for completion
// flags, make everything written for the utterance visible outside the device before the
// flag is raised.  Called by the thread that wrote the row's outputs, or after a
// work-group barrier behind that thread.
__device__ __forceinline__ void finish_row(const DecodeParams &p, int r)
{
    const int b = c.b[r];
    p.tok_len[b] = c.cnt[r];
    if (p.done) __hip_atomic_store(p.done + b, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
}

// RG: row groups (of 4) of a team in the prediction stages; RGJ: row groups a joint step is
// laid out for (its samples never exceed 4 * RGJ); VARIANT: which loop nest; WT: storage of
// the packed weights.
template <int RG, int RGJ, int VARIANT, int WT>
__global__ void __launch_bounds__(kThreads) decode_kernel(const DecodeParams p)
{
    extern __shared__ __align__(16) float dyn_lds[];
    Wg w;
    w.tid = threadIdx.x; w.lane = w.tid & 63;
    // the wave index is the same for all lanes: telling the compiler keeps everything derived
    // from it (task numbers, stream addresses) in scalar registers
    w.wave = __builtin_amdgcn_readfirstlane(w.tid >> 6);
    if (p.spread) { w.rank = blockIdx.x % p.team_size; w.team = blockIdx.x / p.team_size; }
    else { w.team = blockIdx.x % p.n_teams; w.rank = blockIdx.x / p.n_teams; }
    w.jg = w.rank / p.jteam_size; w.jrank = w.rank - w.jg * p.jteam_size;
    Sync sy;
    sy.epoch = 0; sy.jepoch = 0; sy.pepoch = 0; sy.polls = 0;
#ifdef RNNT_PROFILE
    if (w.tid == 0) {
        for (int i = 0; i < 24; ++i) g_prof[i] = 0;
        g_prof_last = wall_clock64();
    }
#endif
    Lds l;
    l.xz = dyn_lds + p.lds_xz; l.red = dyn_lds + p.lds_red; l.c = dyn_lds + p.lds_c;
    l.part = dyn_lds + p.lds_part; l.q = dyn_lds + p.lds_q; l.hc = dyn_lds + p.lds_hc;
    l.tail = dyn_lds + p.lds_tail;
    l.b_pred = dyn_lds + p.lds_bias;
    l.b_out = l.b_pred + 4 * p.gp_max;
    l.b_lstm = l.b_out + 4 * p.gj_max;
    l.s_pred = reinterpret_cast<unsigned char *>(dyn_lds + p.lds_scale);
    l.s_out = l.s_pred + 4 * p.gp_max * scale_blocks(WT, p.spred.kpad);
    l.s_hh = l.s_out + 4 * p.gj_max * scale_blocks(WT, p.sjoint.kpad);
    l.s_ih = l.s_hh + 4 * p.L * p.nu_max * scale_blocks(WT, p.st0.kpad);

    if (w.tid == 0) {
        // XCC_ID hardware register, bits [3:0]
        p.xcc[w.rank * p.n_teams + w.team] = (int)(__builtin_amdgcn_s_getreg((3 << 11) | 20) & 0xf);
    }
    // Rows of this team.  Utterances are ranked by length (longest first, ties by index)
    // and dealt to the teams in serpentine order (0..n-1, n-1..0, ...), so that the sums of
    // the lengths, which is what a team's work grows with, come out even.  Every work-group
    // computes the same assignment from enc_len.
    int R = 0;
    for (int q = 0; q * p.n_teams < p.B; ++q) {
        const int m = ((q & 1) && p.serpentine) ? p.n_teams - 1 - w.team : w.team;
        if (q * p.n_teams + m < p.B) ++R;
    }
    if (R == 0) return;            // the whole team leaves: no barrier is ever entered
    if (w.tid == 0) {
        c.R = R; c.ns = 0; c.bar_ok = 1; c.committed = 0; c.any[0] = 0; c.any[1] = 0;
        c.st_clamped = 0; c.st_overflow = 0;
#pragma unroll
        for (int i = 0; i < kMaxDur; ++i) c.durations[i] = p.durations[i];
    }
    if (w.tid < kMaxRows) {
        const int r = w.tid;
        c.b[r] = 0; c.len[r] = 0; c.t[r] = 0; c.n[r] = 0; c.last[r] = p.blank;
        c.cnt[r] = 0; c.sel[r] = 0; c.active[r] = 0; c.searching[r] = 0;
        c.mask[r] = 1; c.hold_k[r] = 0; c.hold_d[r] = 0; c.hold_v[r] = 0.f; c.emitted[r] = 0;
    }
    __syncthreads();
    for (int b = w.tid; b < p.B; b += kThreads) {
        const int raw = p.enc_len[b];
        if (raw < 0 || raw > p.T) c.st_clamped = 1;
        const int len = min(max(raw, 0), p.T);
        int pos = 0;
        for (int o = 0; o < p.B; ++o) {
            const int lo = min(max(p.enc_len[o], 0), p.T);
            pos += (lo > len || (lo == len && o < b)) ? 1 : 0;
        }
        const int q = pos / p.n_teams, m = pos - q * p.n_teams;
        const int team = ((q & 1) && p.serpentine) ? p.n_teams - 1 - m : m;
        if (team == w.team) { c.b[q] = b; c.len[q] = len; c.active[q] = len > 0; }
    }
    __syncthreads();
    // this rank's slices of the bias vectors
    {
        const int gpa = (p.J + 3) / 4, gja = (p.nout_m + 3) / 4;
        const int gp0 = range_lo(w.rank, p.team_size, gpa), ngp = range_hi(w.rank, p.team_size, gpa) - gp0;
        const int gj0 = range_lo(w.jrank, p.jteam_size, gja), ngj = range_hi(w.jrank, p.jteam_size, gja) - gj0;
        const int hu0 = range_lo(w.rank, p.team_size, p.H), hnu = range_hi(w.rank, p.team_size, p.H) - hu0;
        for (int i = w.tid; i < ngp * 4; i += kThreads)
            l.b_pred[i] = (gp0 * 4 + i < p.J) ? p.b_pred[gp0 * 4 + i] : 0.f;
        for (int i = w.tid; i < ngj * 4; i += kThreads)
            l.b_out[i] = (gj0 * 4 + i < p.nout_m) ? p.b_out[gj0 * 4 + i] : 0.f;
        if (w.jrank < p.n_tail) {
            const int tk = (p.J + 3) & ~3;
            for (int i = w.tid; i < tk; i += kThreads) l.tail[i] = p.w_tail[(long long)w.jrank * tk + i];
        }
        for (int i = w.tid; i < p.L * hnu * 4; i += kThreads) {
            const int layer = i / (hnu * 4), rem = i - layer * hnu * 4;
            l.b_lstm[(layer * p.nu_max) * 4 + rem] = p.bias_l[((long long)layer * p.H + hu0) * 4 + rem];
        }
        if (WT == kWeightFp8Bf16Arith || WT == kWeightFp4Bf16Arith) {
            // table entry [row][b] = the matrix's scale of that row's block b, 1 beyond the matrix
            const int nbp = scale_blocks(WT, p.spred.kpad), nbo = scale_blocks(WT, p.sjoint.kpad);
            const int nbh = scale_blocks(WT, p.st0.kpad);
            const int gbh = scale_blocks_of_matrix(WT, p.H), gbj = scale_blocks_of_matrix(WT, p.J);
            for (int i = w.tid; i < ngp * 4 * nbp; i += kThreads) {
                const int col = gp0 * 4 + i / nbp, b = i % nbp;
                l.s_pred[i] = scale_byte((col < p.J && b < gbh) ? p.sc_pred[(long long)col * gbh + b] : 1.0f);
            }
            for (int i = w.tid; i < ngj * 4 * nbo; i += kThreads) {
                const int col = gj0 * 4 + i / nbo, b = i % nbo;
                l.s_out[i] = scale_byte((col < p.nout_m && b < gbj) ? p.sc_out[(long long)col * gbj + b] : 1.0f);
            }
            for (int i = w.tid; i < p.L * hnu * 4 * nbh; i += kThreads) {
                const int row = i / nbh, b = i % nbh;
                const int layer = row / (hnu * 4), rem = row - layer * hnu * 4;
                l.s_hh[i] = scale_byte(b < gbh ? p.sc_hh[(((long long)layer * p.H + hu0) * 4 + rem) * gbh + b] : 1.0f);
            }
            for (int layer = 1; layer < p.L; ++layer) {
                const int nbi = scale_blocks(WT, p.stl[layer < kMaxLayers ? layer : 0].kpad);
                for (int i = w.tid; i < hnu * 4 * nbi; i += kThreads) {
                    const int rem = i / nbi, b = i % nbi;
                    l.s_ih[layer * hnu * 4 * p.sc_nb_in + i] =
                        scale_byte(b < gbh ? p.sc_ih[(((long long)layer * p.H + hu0) * 4 + rem) * gbh + b] : 1.0f);
                }
            }
        }
    }
    // zero state: c of both selectors, committed h of this rank's units
    const int u0 = range_lo(w.rank, p.team_size, p.H), nu = range_hi(w.rank, p.team_size, p.H) - u0;
    for (int i = w.tid; i < p.L * 2 * p.nu_max * p.rcap; i += kThreads) l.c[i] = 0.f;
    if (p.fast_pred)     // the LDS copies of the hidden vectors: zero state, zero rows beyond R, zero K padding
        for (int i = w.tid; i < 2 * p.L * 4 * p.xstride; i += kThreads) l.hc[i] = 0.f;
    for (int i = w.tid; i < p.L * R * nu; i += kThreads) {
        const int layer = i / (R * nu), rem = i - layer * R * nu;
        const int r = rem / nu, u = rem - r * nu;
        xstore(h_slot(p, w.team, 0, layer, r) + u0 + u, 0.f);
    }
    // Output fill.  A row's outputs are only ever written by one work-group, the one that
    // will emit the row's labels (first rank of the row's joint group): the work-groups of a
    // team sit on different XCDs, whose L2s are not coherent with each other for plain stores,
    // so a fill written by another work-group could reach memory after the labels it was
    // meant to precede.  Within a work-group the barrier below orders fill and labels.
    for (int r = w.jg; r < R; r += p.groups) {
        if (w.jrank != 0) break;
        const long long o = (long long)c.b[r] * p.cap;
        for (int i = w.tid; i < p.cap; i += kThreads) {
            p.tokens[o + i] = -1;
            if (p.frames) p.frames[o + i] = -1;
            if (p.logits) p.logits[o + i] = 0.f;
            if (p.logps) p.logps[o + i] = 0.f;
            if (p.durs) p.durs[o + i] = -1;
        }
    }
    // a failed first barrier skips the loops and reaches the epilogue, which reports it
    bool ok = team_barrier(p, w, sy);
    // empty utterances are complete from the start
    if (ok && w.jrank == 0 && w.tid < R && w.tid % p.groups == w.jg && !c.active[w.tid]) finish_row(p, w.tid);

    long long n_pred = 0, n_joint = 0, n_samples = 0;

    if constexpr (VARIANT == kFrameLooping || VARIANT == kFrameLoopingSingle) {
        // Algorithm 1 on this team's rows.  A joint step also evaluates the next frames of
        // every row with the same g (lookahead); those results stand in for the first joint
        // evaluation of the following frames for as long as no row emits, that is, for as
        // long as no (last_label, hidden) changes: the same values the algorithm would compute.
        int la = p.lookahead;
        if (la * R > RGJ * 4) la = RGJ * 4 / R;      // the host sized RGJ for lookahead * rows
        if (la < 1) la = 1;
        int max_out_len = 0;
        for (int r = 0; r < R; ++r) max_out_len = max(max_out_len, c.len[r]);
        if constexpr (VARIANT == kFrameLoopingSingle) {
            // One utterance per team (the default up to 32 utterances): there are no batch mates
            // to keep in step, so the loop nest reduces to its decisions.  Every thread reads the
            // same results of a joint step and takes the same decisions from them; only an
            // emission, whose state the prediction step reads next, needs a barrier.
            //   t      frame index (Algorithm 1's time_idx), n_sym labels emitted on frame t
            //   window frames [win0, win0 + win_n) have joint results for the current g
            const int len = c.len[0];
            int t = 0, n_sym = 0, win0 = 0, win_n = 0;
            bool need_pred = true;
            while (ok && t < len) {
                if (need_pred) {
                    ok = prediction_step<RG, WT>(p, w, sy, l);
                    if (!ok) break;
                    ++n_pred;
                    need_pred = false;
                    win_n = 0;
                }
                if (t >= win0 + win_n) {
                    const int n_ahead = min(la, len - t);
                    if (w.tid < kMaxSamples) {
                        const int s = w.tid, valid = s < n_ahead;
                        c.s_row[s] = 0; c.s_frame[s] = t + s; c.s_valid[s] = valid;
                        c.s_pidx[s] = valid ? c.b[0] * p.T + t + s : -1;
                        c.s_qoff[s] = 0;
                    }
                    if (w.tid == 0) c.ns = n_ahead;
                    __syncthreads();
                    ok = joint_step<RGJ, WT>(p, w, sy, l);
                    if (!ok) break;
                    ++n_joint; n_samples += n_ahead;
                    win0 = t; win_n = n_ahead;
                }
                // the first label among the window's frames from t on; blanks before it only
                // move the frame index
                const int s = w.lane & (kMaxSamples - 1);
                const bool label = w.lane < win_n && win0 + s >= t && c.s_k[s] != p.blank;
                const unsigned long long m = __ballot(label);
                if (!m) { t = win0 + win_n; n_sym = 0; continue; }
                const int i = __ffsll((long long)m) - 1;
                if (win0 + i > t) { t = win0 + i; n_sym = 0; }
                if (w.tid == 0) emit_row(p, w, 0, c.s_k[i], t, c.s_v[i], c.s_lp[i], 0);
                need_pred = true;
                if (++n_sym == p.S) { ++t; n_sym = 0; }     // max_symbols labels on this frame: move on
                // the emission's state (last label, selector, count) before the prediction step reads it
                __syncthreads();
            }
        } else {
            bool need_pred = true;     // nothing computed yet for (last_label, hidden)
            int flip = 0;              // slot of c.any the next inner step reports in
            int win0 = 0, win_n = 0;   // frames [win0, win0 + win_n) have results for the current g
            for (int time_idx = 0; ok && time_idx < max_out_len; ++time_idx) {
                // Frames the window already covers and on which every row produced a blank change
                // nothing but the frame index: they are passed over in one go (each would run the
                // inner loop once, find all blank and leave).  Every thread reads the same results
                // and takes the same decision.
                if (!need_pred && time_idx > win0 && time_idx < win0 + win_n) {
                    // (every wave looks at all results at once: lane s holds sample s = frame offset
                    // s / R, row s % R, and the first label among the frames from time_idx on decides)
                    int f;
                    {
                        const int s = w.lane & (kMaxSamples - 1), i = s / R, r = s - i * R;
                        const int k = c.s_k[s], len_r = c.len[r];
                        const bool label = w.lane < win_n * R && win0 + i >= time_idx && win0 + i < len_r && k != p.blank;
                        const unsigned long long m = __ballot(label);
                        f = m ? win0 + (__ffsll((long long)m) - 1) / R : win0 + win_n;
                    }
                    if (f > time_idx) {
                        // rows whose frames ran out on the way are complete
                        if (w.rank == 0 && w.tid < R && c.len[w.tid] >= time_idx && c.len[w.tid] < f &&
                            c.len[w.tid] > 0)
                            finish_row(p, w.tid);
                        time_idx = f;
                        if (time_idx >= max_out_len) break;
                    }
                }
                if (w.tid < R) {
                    c.mask[w.tid] = time_idx >= c.len[w.tid];   // a row whose frames have run out starts the frame masked
                    // a row whose frames have run out is complete although the team goes on
                    if (w.rank == 0 && time_idx == c.len[w.tid] && time_idx > 0) finish_row(p, w.tid);
                }
                int symbols_added = 0;
                bool not_blank = true;
                __syncthreads();
                while (ok && not_blank && symbols_added < p.S) {
                    if (need_pred) {
                        // the prediction network's step of Algorithm 1's inner loop; skipped when neither
                        // input changed since the last evaluation (same result)
                        ok = prediction_step<RG, WT>(p, w, sy, l);
                        if (!ok) break;
                        ++n_pred;
                        need_pred = false;
                        win_n = 0;
                    }
                    int off = 0;
                    if (symbols_added == 0 && time_idx >= win0 && time_idx < win0 + win_n) {
                        off = time_idx - win0;
                    } else {
                        const int n_ahead = min(la, max_out_len - time_idx);
                        if (w.tid < kMaxSamples) {
                            const int s = w.tid, i = s / R, r = s - i * R;
                            const int fr = time_idx + i;
                            const int valid = i < n_ahead && (i == 0 ? !c.mask[r] : fr < c.len[r]);
                            c.s_row[s] = r; c.s_frame[s] = fr; c.s_valid[s] = valid;
                            c.s_pidx[s] = valid ? c.b[r] * p.T + fr : -1;
                            c.s_qoff[s] = p.q_in_lds ? (r / p.groups) * p.qstride : r;
                        }
                        if (w.tid == 0) c.ns = R * n_ahead;
                        __syncthreads();
                        ok = joint_step<RGJ, WT>(p, w, sy, l);
                        if (!ok) break;
                        ++n_joint; n_samples += R * n_ahead;
                        win0 = time_idx; win_n = n_ahead;
                    }
                    if (w.tid == 0) {
                        int any = 0;
                        for (int r = 0; r < R; ++r) {
                            if (c.mask[r]) continue;
                            const int k = c.s_k[off * R + r];
                            if (k == p.blank) { c.mask[r] = 1; }          // a blank masks the row for the rest of the frame
                            else { emit_row(p, w, r, k, time_idx, c.s_v[off * R + r], c.s_lp[off * R + r], 0); any = 1; }
                        }
                        c.any[flip] = any;
                    }
                    __syncthreads();
                    // the next inner step reports in the other slot, and this slot is written again
                    // only after the barrier of that step: no second barrier is needed here
                    not_blank = c.any[flip] != 0;
                    flip ^= 1;
                    need_pred = need_pred || not_blank;
                    symbols_added += 1;
                }
            }
        }
    } else {
        // Label looping (RNN-T and TDT).  The team runs the prediction network for all its
        // rows; each of its joint groups then searches the next label of its own rows (row r
        // belongs to group r mod groups) without waiting for the other groups, and publishes
        // what the next prediction step needs of them: last label, state selector, activity.
        const bool tdt = p.D > 0;
        const int G = p.groups, g = w.jg;
        const int rj = R > g ? (R - g + G - 1) / G : 0;      // rows of this group
        int la = p.lookahead;
        if (rj > 0 && la * rj > RGJ * 4) la = RGJ * 4 / rj;   // the host sized RGJ for lookahead * rows
        if (la < 1) la = 1;
        unsigned outer = 0;
        // The loop control runs in the first wave only (lane j looks after the group's row j),
        // between two work-group barriers; the other waves read its decisions from c.f_*.
        // Samples of the next joint step: `la` consecutive frames of every searching row.
        auto set_up_samples = [&]() {
            const int s = w.lane, j = s / la, i = s - j * la;
            int valid = 0, fr = 0, row = 0;
            if (s < kMaxSamples && j < rj) {
                row = g + j * G; fr = c.t[row] + i;
                valid = c.searching[row] && fr < c.len[row];
            }
            if (s < kMaxSamples) {
                c.s_row[s] = row; c.s_frame[s] = fr; c.s_valid[s] = valid;
                c.s_pidx[s] = valid ? c.b[row] * p.T + fr : -1;
                c.s_qoff[s] = p.q_in_lds ? (row / G) * p.qstride : row;
            }
            const unsigned long long vmask = __ballot(valid != 0);
            if (w.lane == 0) { c.ns = rj * la; n_samples += __popcll(vmask); }
        };
        if (w.wave == 0) {
            int act = 0;
            if (w.lane < R) act = c.active[w.lane];
            if (w.lane == 0) { c.f_any_active = __ballot(act != 0) != 0ull; c.f_need_pred = 1; }
        }
        __syncthreads();
        while (ok && c.f_any_active) {
            ++outer;
            if (c.f_need_pred) {
                ok = prediction_step<RG, WT>(p, w, sy, l);
                if (!ok) break;
                ++n_pred;
            } else {
                // Every iteration meets the whole team once, here or inside the prediction
                // step: no work-group can then be more than one iteration behind another, which
                // is what the two parity slots of the row-state exchange below rely on.
                ok = team_barrier(p, w, sy);
                if (!ok) break;
            }
            // A search is cut off after search_steps joint steps (0: never): rows that have
            // found their label go on to the next prediction step instead of waiting for a row
            // in a long run of blanks; that row keeps its state through the step (prediction()
            // of unchanged inputs gives the same g) and searches on afterwards.  When no row
            // of the team emitted, nothing changed and the prediction step is skipped.
            int steps_left = p.search_steps > 0 ? p.search_steps : 0x7fffffff;
            if (w.wave == 0) {
                int searching = 0;
                if (w.lane < R) {
                    searching = (w.lane % G == g) && c.active[w.lane];
                    c.searching[w.lane] = searching; c.emitted[w.lane] = 0;
                }
                const bool any = __ballot(searching != 0) != 0ull;
                if (w.lane == 0) c.f_any_searching = any;
                if (any) set_up_samples();
            }
            __syncthreads();
            while (ok && c.f_any_searching && steps_left-- > 0) {
                ok = joint_step<RGJ, WT>(p, w, sy, l);
                if (!ok) break;
                ++n_joint;
                if (w.wave == 0 && !tdt && p.VT == p.V1) {
                    // Plain transducer: a blank moves on by one frame, so the walk is the first
                    // non-blank result among the frames the row still has.  Every lane reads one
                    // sample's result; lane j then takes row j's part of the ballot.
                    // (the read is unconditional: lanes past the samples read a slot that exists)
                    const int mine = c.s_k[w.lane & (kMaxSamples - 1)];
                    const unsigned long long labels = __ballot(w.lane < c.ns && mine != p.blank);
                    int still = 0;
                    if (w.lane < rj && c.searching[g + w.lane * G]) {
                        const int j = w.lane, r = g + j * G;
                        const int t0 = c.t[r], avail = min(la, c.len[r] - t0);
                        const unsigned long long seg = (labels >> (j * la)) & ((1ull << avail) - 1ull);
                        const int pos = seg ? __ffsll((long long)seg) - 1 : avail;
                        if (pos > 0) c.n[r] = 0;
                        c.t[r] = t0 + pos;
                        still = 1;
                        if (seg) {
                            const int s = j * la + pos;
                            c.hold_k[r] = c.s_k[s]; c.hold_v[r] = c.s_v[s]; c.hold_lp[r] = c.s_lp[s]; c.hold_d[r] = 0;
                            c.searching[r] = 0; still = 0;
                        } else if (t0 + pos >= c.len[r]) {
                            c.searching[r] = 0; c.active[r] = 0; still = 0;
                            if (w.jrank == 0) finish_row(p, r);
                        }
                    }
                    const bool any = __ballot(still != 0) != 0ull;
                    if (w.lane == 0) c.f_any_searching = any;
                    if (any && steps_left > 0) set_up_samples();
                } else if (w.wave == 0) {
                    // lane j walks the results of the group's row j in frame order
                    int still = 0;
                    if (w.lane < rj && c.searching[g + w.lane * G]) {
                        const int j = w.lane, r = g + j * G;
                        int pos = 0, found = 0;
                        while (pos < la && c.t[r] + pos < c.len[r]) {
                            const int s = j * la + pos;
                            const int k = c.s_k[s];
                            const int dval = tdt ? c.durations[c.s_d[s]] : 0;
                            if (k >= p.V1) {
                                // a big blank of a multi-blank model: skip its span of frames
                                pos += max(c.durations[k - p.V1], 1);
                                c.n[r] = 0;
                            } else if (k == p.blank) {
                                pos += tdt ? max(dval, 1) : 1;
                                c.n[r] = 0;
                            } else {
                                found = 1;
                                c.hold_k[r] = k; c.hold_v[r] = c.s_v[s]; c.hold_lp[r] = c.s_lp[s]; c.hold_d[r] = dval;
                                break;
                            }
                        }
                        c.t[r] += pos;
                        still = 1;
                        if (found) { c.searching[r] = 0; still = 0; }
                        else if (c.t[r] >= c.len[r]) {
                            c.searching[r] = 0; c.active[r] = 0; still = 0;
                            if (w.jrank == 0) finish_row(p, r);
                        }
                    }
                    const bool any = __ballot(still != 0) != 0ull;
                    if (w.lane == 0) c.f_any_searching = any;
                    if (any && steps_left > 0) set_up_samples();
                }
                __syncthreads();
            }
            if (!ok) break;
            PROF_MARK(w, 16);
            if (w.wave == 0) {
                // rows that hold a label emit it and move on
                if (w.lane < rj && c.active[g + w.lane * G] && !c.searching[g + w.lane * G]) {
                    const int r = g + w.lane * G;
                    const int dval = c.hold_d[r];
                    emit_row(p, w, r, c.hold_k[r], c.t[r], c.hold_v[r], c.hold_lp[r], dval);
                    if (tdt && dval > 0) { c.t[r] += dval; c.n[r] = 0; }
                    else { c.n[r] += 1; if (c.n[r] == p.S) { c.t[r] += 1; c.n[r] = 0; } }
                    c.active[r] = c.t[r] < c.len[r];
                    c.emitted[r] = 1;
                    if (!c.active[r] && w.jrank == 0) finish_row(p, r);
                }
                if (G > 1) {
                    // tell the other groups about this group's rows, learn about theirs
                    if (w.jrank == 0 && w.lane < rj) {
                        const int r = g + w.lane * G;
                        const unsigned payload = ((unsigned)c.last[r] & 0xffffu) |
                                                 ((unsigned)c.sel[r] << 16) | ((unsigned)c.active[r] << 17) |
                                                 ((unsigned)c.emitted[r] << 18);
                        // two slots per row, by parity of the iteration: a group that runs ahead
                        // writes the other slot, and reaches this one again only two iterations
                        // later, after a team-wide meeting that every work-group enters only when
                        // it has read this one
                        xstore64(p.rowx + ((long long)w.team * 2 + (outer & 1u)) * kMaxRows + r,
                                 ((unsigned long long)outer << 32) | payload);
                    }
                    // (a row that has ended stays ended: nothing more to learn about it)
                    if (w.lane < R && w.lane % G != g && c.active[w.lane]) {
                        const int r = w.lane;
                        const unsigned long long *slot =
                            p.rowx + ((long long)w.team * 2 + (outer & 1u)) * kMaxRows + r;
                        unsigned spins = 0;
                        unsigned long long v = xload64(slot);
                        while ((unsigned)(v >> 32) != outer) {
                            ++spins;
                            if ((spins & 127u) == 0 &&
                                __hip_atomic_load(p.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) {
                                c.bar_ok = 0;
                                break;
                            }
                            if (spins > p.spin_limit) {
                                __hip_atomic_store(p.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                c.bar_ok = 0;
                                break;
                            }
                            __builtin_amdgcn_s_sleep(1);
                            v = xload64(slot);
                        }
                        sy.polls += spins;
                        const unsigned payload = (unsigned)v;
                        c.last[r] = (int)(payload & 0xffffu);
                        c.sel[r] = (int)((payload >> 16) & 1u);
                        c.active[r] = (int)((payload >> 17) & 1u);
                        c.emitted[r] = (int)((payload >> 18) & 1u);
                    }
                }
                // the wave's own LDS writes above are visible to its lanes in program order
                int act = 0, emi = 0;
                if (w.lane < R) { act = c.active[w.lane]; emi = c.emitted[w.lane]; }
                const bool any_act = __ballot(act != 0) != 0ull, any_emi = __ballot(emi != 0) != 0ull;
                if (w.lane == 0) { c.f_any_active = any_act; c.f_need_pred = any_emi; }
            }
            __syncthreads();
            ok = c.bar_ok != 0;
            PROF_MARK(w, 19);
        }
    }
    // epilogue
    __syncthreads();
    if (w.jrank == 0 && w.tid < R && w.tid % p.groups == w.jg) finish_row(p, w.tid);
    if (w.jrank == 0 && w.tid == 0) {
        int st = (c.st_clamped ? 1 : 0) | (c.st_overflow ? 2 : 0);
        if (!ok) st |= 4;
        if (st) __hip_atomic_fetch_or(as_global(p.status), st, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (w.rank == 0 && w.tid == 0) {
        long long *sp = p.stats + (long long)w.team * kStatStride;
        // (added: the launches of one call share the counters, the reset kernel zeroes them first)
        sp[kStatPred] += n_pred; sp[kStatJoint] += n_joint; sp[kStatSamples] += n_samples;
        sp[kStatPolls] += sy.polls;
#ifdef RNNT_PROFILE
        for (int i = 0; i < 24; ++i) sp[kStatCount + i] += g_prof[i];
#endif
    } else if (!ok && w.tid == 0) {
        __hip_atomic_fetch_or(as_global(p.status), 4, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}


template <int RG, int RGJ, int VARIANT, int WT>
hipError_t launch_one(const DecodeParams &p, hipStream_t stream)
{
    const void *fn = reinterpret_cast<const void *>(&decode_kernel<RG, RGJ, VARIANT, WT>);
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)p.lds_bytes);
    if (e != hipSuccess) return e;
    DecodeParams pc = p;
    void *args[] = {&pc};
    // The cooperative launch guarantees that all work-groups are resident together, which
    // the team barriers rely on.  An engine created with RNNT_FLAG_PLAIN_LAUNCH uses an
    // ordinary launch instead (the grid is one work-group per compute unit, so on an
    // otherwise idle device it is resident too, and every wait in the kernel is bounded).
    const dim3 grid(p.n_teams * p.team_size), block(kThreads);
    if (p.plain_launch) return hipLaunchKernel(fn, grid, block, args, p.lds_bytes, stream);
    return hipLaunchCooperativeKernel(fn, grid, block, args, p.lds_bytes, stream);
}

// Launch for one loop nest and one prediction row-group count; rgj (1, 2, 4 or 8) picks the
// joint-step layout.
template <int RG, int VARIANT, int WT>
hipError_t launch_variant(const DecodeParams &p, int rgj, hipStream_t stream)
{
    switch (rgj) {
    case 1: return launch_one<RG, 1, VARIANT, WT>(p, stream);
    case 2: return launch_one<RG, 2, VARIANT, WT>(p, stream);
    case 4: return launch_one<RG, 4, VARIANT, WT>(p, stream);
    default: return launch_one<RG, 8, VARIANT, WT>(p, stream);
    }
}

}  // namespace
}  // namespace rnnt
