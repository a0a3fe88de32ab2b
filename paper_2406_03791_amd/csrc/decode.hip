// Host side of the decode launch: the reset kernel and the choice of the decode kernel
// instance (the kernels themselves are in decode_impl.h, instantiated by decode_*.hip).
#include "engine.h"

namespace rnnt {

// launch_decode_<nest><row groups>_<storage>: one per instantiation unit (decode_inst.hip)
#define RNNT_DECLARE_LAUNCH(name) \
    hipError_t name(const DecodeParams &p, int rgj, hipStream_t stream)
#define RNNT_DECLARE_NEST(wt)                                                            \
    RNNT_DECLARE_LAUNCH(launch_decode_f1_##wt); RNNT_DECLARE_LAUNCH(launch_decode_f2_##wt); \
    RNNT_DECLARE_LAUNCH(launch_decode_f4_##wt); RNNT_DECLARE_LAUNCH(launch_decode_l1_##wt); \
    RNNT_DECLARE_LAUNCH(launch_decode_l2_##wt); RNNT_DECLARE_LAUNCH(launch_decode_l4_##wt); \
    RNNT_DECLARE_LAUNCH(launch_decode_s1_##wt)
RNNT_DECLARE_NEST(f32); RNNT_DECLARE_NEST(bf16); RNNT_DECLARE_NEST(fp8); RNNT_DECLARE_NEST(bf16a);
RNNT_DECLARE_NEST(fp8a);
RNNT_DECLARE_NEST(fp4a);
#undef RNNT_DECLARE_NEST
#undef RNNT_DECLARE_LAUNCH

// Clears what must start at zero for a launch: barrier counters, abort flag and the tagged
// argmax partials and row states (a tag left by the previous launch must not look current);
// the status word only in the first launch of a call and the statistics only in the first
// launch that uses their buffer.
__global__ void reset_kernel(unsigned *bar, int n_bar, unsigned *abort_flag, int *status, int zero_status, int zero_stats,
                             long long *stats, int n_stats, unsigned long long *part,
                             unsigned long long *dpart, unsigned long long *lpart, int n_part,
                             unsigned long long *rowx, int n_rowx, unsigned long long *xh, int n_xh,
                             unsigned long long *xq, int n_xq)
{
    const int i0 = blockIdx.x * blockDim.x + threadIdx.x;
    if (i0 < n_bar) bar[i0] = 0u;
    if (i0 < n_stats && zero_stats) stats[i0] = 0;
    if (i0 < n_part) { part[i0] = 0ull; dpart[i0] = 0ull; lpart[i0] = 0ull; }
    if (i0 < n_rowx) rowx[i0] = 0ull;
    if (i0 == 0) { *abort_flag = 0u; if (zero_status) *status = 0; }
    // the tagged hidden-vector and q words (the larger arrays): grid-stride
    for (int i = i0; i < n_xh; i += gridDim.x * blockDim.x) xh[i] = 0ull;
    for (int i = i0; i < n_xq; i += gridDim.x * blockDim.x) xq[i] = 0ull;
}

hipError_t launch_decode(const DecodeParams &p, bool zero_status, bool zero_stats, hipStream_t stream)
{
    const int n_bar = p.n_teams * 32, n_stats = p.n_teams * kStatStride;
    const int n_part = p.n_teams * p.groups * 2 * kMaxSamples * p.jteam_size;
    int n = n_bar > n_stats ? n_bar : n_stats;
    n = n > n_part ? n : n_part;
    const int n_xh = p.fast_pred ? p.n_teams * p.L * kMaxRows * p.H : 0;
    const int n_xq = p.fast_pred ? p.n_teams * kMaxRows * p.J : 0;
    int blocks = (n + 255) / 256;
    if (p.fast_pred && blocks < 256) blocks = 256;
    hipLaunchKernelGGL(reset_kernel, dim3(blocks), dim3(256), 0, stream, p.bar, n_bar,
                       p.abort_flag, p.status, zero_status ? 1 : 0, zero_stats ? 1 : 0, p.stats, n_stats, p.part, p.dpart, p.lpart, n_part, p.rowx,
                       p.n_teams * 2 * kMaxRows, p.xh, n_xh, p.xq, n_xq);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // kernels are instantiated per loop nest, per row-group count of the prediction stages
    // and per row-group count of the joint step
    const int rows = (p.B + p.n_teams - 1) / p.n_teams;
    const int rg = pred_row_groups(rows);
    const int rows_j = (rows + p.groups - 1) / p.groups;
    const int samples = rows_j * p.lookahead;
    const int rgj = joint_row_groups(samples);
    const int rgi = rg <= 1 ? 0 : (rg <= 2 ? 1 : 2);
    // the LDS layout of the call was planned for rg_planned row groups and samples_cap samples: an instance
    // that assumes more would write outside its regions
    if (rows > kMaxRows || rg > p.rg_planned || samples > p.samples_cap) return hipErrorInvalidValue;
    typedef hipError_t (*Launch)(const DecodeParams &, int, hipStream_t);
    static const Launch table[kWeightTypes][2][3] = {
        {{launch_decode_f1_f32, launch_decode_f2_f32, launch_decode_f4_f32},
         {launch_decode_l1_f32, launch_decode_l2_f32, launch_decode_l4_f32}},
        {{launch_decode_f1_bf16, launch_decode_f2_bf16, launch_decode_f4_bf16},
         {launch_decode_l1_bf16, launch_decode_l2_bf16, launch_decode_l4_bf16}},
        {{launch_decode_f1_fp8, launch_decode_f2_fp8, launch_decode_f4_fp8},
         {launch_decode_l1_fp8, launch_decode_l2_fp8, launch_decode_l4_fp8}},
        {{launch_decode_f1_bf16a, launch_decode_f2_bf16a, launch_decode_f4_bf16a},
         {launch_decode_l1_bf16a, launch_decode_l2_bf16a, launch_decode_l4_bf16a}},
        {{launch_decode_f1_fp8a, launch_decode_f2_fp8a, launch_decode_f4_fp8a},
         {launch_decode_l1_fp8a, launch_decode_l2_fp8a, launch_decode_l4_fp8a}},
        {{launch_decode_f1_fp4a, launch_decode_f2_fp4a, launch_decode_f4_fp4a},
         {launch_decode_l1_fp4a, launch_decode_l2_fp4a, launch_decode_l4_fp4a}}};
    if (p.wt < 0 || p.wt >= kWeightTypes) return hipErrorInvalidValue;
    // Algorithm 1 with one utterance per team has an instance of its own.  For a single row the
    // label-looping schedule of an RNN-T is the same sequence of prediction and joint steps
    // (the two differ in how a batch is kept in step), so such teams use it too; TDT and
    // multi-blank models have rules of their own for the frame index and stay with theirs.
    static const Launch single[kWeightTypes] = {launch_decode_s1_f32, launch_decode_s1_bf16, launch_decode_s1_fp8,
                                                launch_decode_s1_bf16a, launch_decode_s1_fp8a, launch_decode_s1_fp4a};
    const bool plain_label = p.variant == kLabelLooping && p.D == 0 && p.VT == p.V1 && p.groups == 1;
    if ((p.variant == kFrameLooping || plain_label) && rows == 1) return single[p.wt](p, rgj, stream);
    return table[p.wt][p.variant == kFrameLooping ? 0 : 1][rgi](p, rgj, stream);
}

}  // namespace rnnt
