// Work decomposition shared by the host-side weight packer and the decode kernel.
//
// A team of `ts` work-groups decodes a subset of the batch.  Every dense stage
// of a step (LSTM gates, prediction-side joint projection, joint output
// projection) is a small-M product  out[rows, N] = x[rows, K] * W[N, K]^T.  Its
// N outputs are cut into groups of 4 columns (for the LSTM: the four gates of
// one hidden unit) that are dealt to the ranks of the team in contiguous
// ranges; inside a rank each group is cut again along K into `nks` slices.
// One (group, K-slice) pair is a task; a task runs on one 4-lane block of a
// wavefront with v_mfma_f32_4x4x1 (4 rows x 4 columns per block, 16 blocks per
// wave, kBlocksPerWg blocks per work-group).  Tasks beyond that go to further
// "slots", processed one after the other.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#define RNNT_HD __host__ __device__

namespace rnnt {

constexpr int kThreads = 512;        // threads per work-group (8 wavefronts, 2 per SIMD)
constexpr int kWaves = kThreads / 64;
constexpr int kBlocksPerWg = kWaves * 16;   // 4-lane MFMA blocks per work-group
constexpr int kMaxLayers = 4;
constexpr int kMaxDur = 8;
constexpr int kMaxRows = 16;         // utterances per team
constexpr int kMaxSamples = 32;      // (utterance, frame) pairs per joint step
constexpr int kStepUnroll = 4;       // weight loads (16 bytes per lane) per software-pipeline batch
constexpr int kAheadSteps = 4 * kStepUnroll;   // at least the loads a lane keeps in flight (the packed buffers' end padding)

// Storage of the packed weights: fp32 (4 K values per 16-byte load), bf16 (8 per load) or
// fp8 in the OCP e4m3 format (16 per load).  With the three storage types the arithmetic is
// fp32 on the stored values (a stored weight is widened before it is used, and the storage is
// lossless or refused).  kWeightBf16Arith is the bfloat16 mode: the weights are rounded to
// bf16 and stored as such, and every vector that enters a product is rounded to bf16 too;
// products of two bf16 values are exact in fp32 and the sums stay fp32.
// kWeightFp8Bf16Arith is the bfloat16 mode with its weights stored as e4m3 (lossless or refused):
// a stored weight is widened to bf16, which holds every e4m3 value, on its way to the bf16 MFMA,
// and multiplied by its row's power-of-two scale in the same instruction.
// kWeightFp4Bf16Arith: the same with 4-bit codes in the OCP e2m1 format (32 per load) and one
// power-of-two scale per kScaleBlock consecutive K values of a row.
enum WeightType { kWeightF32 = 0, kWeightBf16 = 1, kWeightFp8 = 2, kWeightBf16Arith = 3, kWeightFp8Bf16Arith = 4,
                  kWeightFp4Bf16Arith = 5, kWeightTypes = 6 };
RNNT_HD constexpr bool is_bf16_arith(int wt)
{
    return wt == kWeightBf16Arith || wt == kWeightFp8Bf16Arith || wt == kWeightFp4Bf16Arith;
}
RNNT_HD constexpr int k_per_load(int wt)
{
    return wt == kWeightFp4Bf16Arith ? 32
         : ((wt == kWeightFp8 || wt == kWeightFp8Bf16Arith) ? 16 : ((wt == kWeightBf16 || wt == kWeightBf16Arith) ? 8 : 4));
}
// K values that share a scale in the 4-bit form: the K values of one software-pipeline batch of
// a lane (kStepUnroll loads of 32), so a K slice of a task is a whole number of blocks and a
// lane changes its scale only between batches.
constexpr int kScaleBlock = kStepUnroll * 32;
// Scales a weight row of a stage has in LDS: one per block of the padded K in the 4-bit form,
// one per row with e4m3 codes.
RNNT_HD constexpr int scale_blocks(int wt, int kpad) { return wt == kWeightFp4Bf16Arith ? kpad / kScaleBlock : 1; }
// Scales per row of a matrix with K columns as the engine keeps them in device memory.
RNNT_HD constexpr int scale_blocks_of_matrix(int wt, int K)
{
    return wt == kWeightFp4Bf16Arith ? (K + kScaleBlock - 1) / kScaleBlock : 1;
}

// Floats between the partial sums of consecutive tasks in LDS: 16 per row group plus a pad that
// spreads the readers (one lane per output group, so a stride of whole multiples of 16 floats
// would put all of them on two banks).
RNNT_HD inline int red_task_stride(int rg) { return rg * 16 + 4; }

// Row groups (of 4 rows) the prediction stages of a team with `rows` utterances are compiled
// for: the kernels are instantiated for 1, 2 and 4 groups.  The LDS layout (activation rows,
// stride of the partial sums) has to be sized for this number, not for ceil(rows / 4).
RNNT_HD inline int pred_row_groups(int rows)
{
    const int rg = (rows + 3) / 4;
    return rg <= 1 ? 1 : (rg <= 2 ? 2 : 4);
}
// Row groups a joint step of `samples` (utterance, frame) pairs is compiled for: 1, 2, 4 or 8.
RNNT_HD inline int joint_row_groups(int samples)
{
    return samples <= 4 ? 1 : (samples <= 8 ? 2 : (samples <= 16 ? 4 : 8));
}

// Contiguous share of n items owned by `rank` out of `ts`.
RNNT_HD inline int range_lo(int rank, int ts, int n) { return (int)(((int64_t)rank * n) / ts); }
RNNT_HD inline int range_hi(int rank, int ts, int n) { return (int)(((int64_t)(rank + 1) * n) / ts); }

struct StagePlan {
    int K;          // input length in floats
    int nks;        // K slices per group
    int nsteps;     // 16-byte loads per lane and task (multiple of kStepUnroll)
    int slots;      // passes over the 128 blocks
    int kper;       // K values per load (4: fp32 weights, 8: bf16, 16: fp8, 32: fp4)
    int kpad;       // nks * nsteps * kper: padded input length
    int64_t rank_stride;   // 16-byte elements of packed weights per rank
};

// Steps a pass over the blocks costs beyond its loads (the partial sums are written out and the
// next pass's tasks are set up), in units of one load step: the weight given to the number of
// passes when the K slicing is chosen.
constexpr int kPassOverheadSteps = 8;

// groups_max: largest number of groups any rank owns in this stage.
// Picks the number of K slices per group: groups_max * nks tasks run in passes ("slots") of
// kBlocksPerWg tasks, a pass takes as long as its nsteps loads, so the choice minimises
// slots * (nsteps + overhead) while the zero padding of K (slices are whole multiples of
// kStepUnroll steps) stays below 1/8.  Ties go to fewer slices (fewer partial sums to add).
// single_pass_only restricts stages with more groups than blocks to unsliced tasks, which
// needs the least LDS for partial sums (the engine falls back to it when LDS is short).
inline StagePlan make_stage_plan(int K, int groups_max, int wt = kWeightF32,
                                 bool single_pass_only = false)
{
    StagePlan p{};
    p.K = K;
    p.kper = k_per_load(wt);
    const int k4 = (K + p.kper - 1) / p.kper;      // loads needed to cover K
    if (groups_max < 1) groups_max = 1;
    auto steps_for = [&](int nks) {
        int n = (k4 + nks - 1) / nks;
        return ((n + kStepUnroll - 1) / kStepUnroll) * kStepUnroll;
    };
    const int cap_k = k4 / kStepUnroll > 0 ? k4 / kStepUnroll : 1;
    int best = 1;
    long best_cost = -1;
    for (int nks = 1; nks <= cap_k; ++nks) {
        const int tasks = groups_max * nks;
        if (single_pass_only && nks > 1 && tasks > kBlocksPerWg) break;
        const int kpad4 = nks * steps_for(nks);
        if (nks > 1 && kpad4 * 8 > k4 * 9) continue;
        const int slots = (tasks + kBlocksPerWg - 1) / kBlocksPerWg;
        const long cost = (long)slots * (steps_for(nks) + kPassOverheadSteps);
        if (best_cost < 0 || cost < best_cost) { best_cost = cost; best = nks; }
    }
    p.nks = best;
    p.slots = (groups_max * best + kBlocksPerWg - 1) / kBlocksPerWg;
    p.nsteps = steps_for(p.nks);
    p.kpad = p.nks * p.nsteps * p.kper;
    p.rank_stride = (int64_t)p.slots * kWaves * p.nsteps * 64;
    return p;
}

// The joint output stage of a joint group of `tj` ranks.  When the output width NOUT is a few
// columns more than a whole number of 4-column groups per rank (1024 labels + blank over 8
// ranks: 257 groups), that extra group costs every rank a coarser K slicing.  Then the MFMA
// part covers the nout_m columns that divide evenly and the n_tail columns after them, at
// most one per rank (rank i takes column nout_m + i), are computed with plain multiply-adds.
// Chosen when its cost, with the tail priced at a few load steps, is below the plain plan's.
struct JointSplit {
    int nout_m;      // columns of the MFMA part (NOUT when there is no tail)
    int n_tail;      // columns computed outside it
    StagePlan plan;  // plan of the MFMA part, for the rank with the most groups
};
constexpr int kTailCostSteps = 4;
inline JointSplit plan_joint_stage(int NOUT, int J, int tj, int wt, bool single_pass_only)
{
    auto cost = [](const StagePlan &pl) { return (long)pl.slots * (pl.nsteps + kPassOverheadSteps); };
    const int groups = (NOUT + 3) / 4, groups_max = (groups + tj - 1) / tj;
    JointSplit js{NOUT, 0, make_stage_plan(J, groups_max, wt, single_pass_only)};
    const int per = 4 * tj, even = (NOUT / per) * per, tail = NOUT - even;
    if (even > 0 && tail > 0 && tail <= tj) {
        const StagePlan pl = make_stage_plan(J, even / per, wt, single_pass_only);
        if (cost(pl) + kTailCostSteps < cost(js.plan)) js = JointSplit{even, tail, pl};
    }
    return js;
}

}  // namespace rnnt
