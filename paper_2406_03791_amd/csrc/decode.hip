// Host side of the decode launch: the reset kernel and the choice of the decode kernel
// instance (the kernels themselves are in decode_impl.h, instantiated by decode_*.hip).
#include "engine.h"

namespace rnnt {

hipError_t launch_decode_f1(const DecodeParams &p, int rgj, hipStream_t stream);
hipError_t launch_decode_f2(const DecodeParams &p, int rgj, hipStream_t stream);
hipError_t launch_decode_f4(const DecodeParams &p, int rgj, hipStream_t stream);
hipError_t launch_decode_l1(const DecodeParams &p, int rgj, hipStream_t stream);
hipError_t launch_decode_l2(const DecodeParams &p, int rgj, hipStream_t stream);
hipError_t launch_decode_l4(const DecodeParams &p, int rgj, hipStream_t stream);

// Clears what must start at zero for a call: barrier counters, abort flag, status, stats and
// the tagged argmax partials and row states (a tag left by the previous call must not look
// current).
__global__ void reset_kernel(unsigned *bar, int n_bar, unsigned *abort_flag, int *status,
                             long long *stats, int n_stats, unsigned long long *part,
                             unsigned long long *dpart, int n_part, unsigned long long *rowx,
                             int n_rowx)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_bar) bar[i] = 0u;
    if (i < n_stats) stats[i] = 0;
    if (i < n_part) { part[i] = 0ull; dpart[i] = 0ull; }
    if (i < n_rowx) rowx[i] = 0ull;
    if (i == 0) { *abort_flag = 0u; *status = 0; }
}

hipError_t launch_decode(const DecodeParams &p, hipStream_t stream)
{
    const int n_bar = p.n_teams * 32, n_stats = p.n_teams * kStatStride;
    const int n_part = p.n_teams * p.groups * 2 * kMaxSamples * p.jteam_size;
    int n = n_bar > n_stats ? n_bar : n_stats;
    n = n > n_part ? n : n_part;
    hipLaunchKernelGGL(reset_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, p.bar, n_bar,
                       p.abort_flag, p.status, p.stats, n_stats, p.part, p.dpart, n_part, p.rowx,
                       p.n_teams * 2 * kMaxRows);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // kernels are instantiated per loop nest, per row-group count of the prediction stages
    // and per row-group count of the joint step
    const int rows = (p.B + p.n_teams - 1) / p.n_teams;
    const int rg = (rows + 3) / 4;
    const int rows_j = (rows + p.groups - 1) / p.groups;
    const int samples = rows_j * p.lookahead;
    const int rgj = samples <= 4 ? 1 : (samples <= 8 ? 2 : (samples <= 16 ? 4 : 8));
    if (p.variant == kFrameLooping) {
        if (rg <= 1) return launch_decode_f1(p, rgj, stream);
        if (rg <= 2) return launch_decode_f2(p, rgj, stream);
        return launch_decode_f4(p, rgj, stream);
    }
    if (rg <= 1) return launch_decode_l1(p, rgj, stream);
    if (rg <= 2) return launch_decode_l2(p, rgj, stream);
    return launch_decode_l4(p, rgj, stream);
}

}  // namespace rnnt
