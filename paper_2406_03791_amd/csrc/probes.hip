// Microbenchmarks of what bounds the decode kernel on this device, exported through the C ABI
// (rnnt_probe_*) so that bench.py --probes can print them and profiles/ can keep them:
//   * stream:   how fast the compute units read a weight slice that stays in their XCD's L2
//               (the decode kernel's situation), and how fast they stream from HBM;
//   * exchange: what one all-to-all hand-over of a vector costs inside a team of work-groups,
//               with a counter barrier and with tagged words;
//   * mfma:     the fp32 matrix rate of the two MFMA shapes the library uses.
// None of this is on the decode path.
#include "../../include/rnnt_greedy.h"

#include <hip/hip_runtime.h>

#include "engine.h"

#include <algorithm>
#include <cstdint>
#include <vector>

namespace {

constexpr int kT = 512;

#define PROBE_TRY(expr)                                            \
    do {                                                           \
        hipError_t e_ = (expr);                                    \
        if (e_ != hipSuccess) return rnnt::hip_fail(e_, #expr);    \
    } while (0)

// ---- stream ---------------------------------------------------------------------------------
// Work-group i reads chunk (i % n_chunks) of the buffer `rounds` times with 16-byte loads, two
// batches of four in flight per lane, like the decode kernel's weight stream.
__global__ void __launch_bounds__(kT) stream_kernel(const float4 *buf, long long chunk_f4, int n_chunks,
                                                    int rounds, float *sink)
{
    const float4 *p = buf + (long long)(blockIdx.x % n_chunks) * chunk_f4;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int r = 0; r < rounds; ++r)
        for (long long i = threadIdx.x; i + 7 * kT < chunk_f4; i += 8 * kT) {
            float4 q[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) q[u] = p[i + u * kT];
#pragma unroll
            for (int u = 0; u < 8; ++u) { acc.x += q[u].x; acc.y += q[u].y; acc.z += q[u].z; acc.w += q[u].w; }
        }
    if (acc.x + acc.y + acc.z + acc.w == 12345.678f) sink[blockIdx.x] = acc.x;   // keeps the loads alive
}

// ---- exchange -------------------------------------------------------------------------------
struct XParams {
    float *buf;                    // [2][n_teams][len]  (barrier mode)
    unsigned long long *words;     // [2][n_teams][len]  (tagged mode; two buffers, by parity of the round:
                                   // nobody is more than one round ahead of the slowest work-group)
    unsigned *ctr;                 // one counter per team, 128 bytes apart
    unsigned *abort_flag;
    float *out;
    int n_teams, team_size, len, iters, tagged;
    unsigned spin_limit;
};

__global__ void __launch_bounds__(kT) exchange_kernel(const XParams a)
{
    __shared__ float lds[4096];
    __shared__ int ok_s;
    const int rank = blockIdx.x % a.team_size, team = blockIdx.x / a.team_size;   // ranks spread over the XCDs
    const int lo = (int)((long long)rank * a.len / a.team_size), hi = (int)((long long)(rank + 1) * a.len / a.team_size);
    float acc = 0.f;
    for (int it = 1; it <= a.iters; ++it) {
        if (a.tagged) {
            unsigned long long *wd = a.words + ((long long)(it & 1) * a.n_teams + team) * a.len;
            for (int i = lo + threadIdx.x; i < hi; i += kT)
                __hip_atomic_store(wd + i, ((unsigned long long)it << 32) | (unsigned)(it + i), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            for (int i = threadIdx.x; i < a.len; i += kT) {
                unsigned spins = 0;
                unsigned long long v = __hip_atomic_load(wd + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                while ((unsigned)(v >> 32) != (unsigned)it) {
                    if (++spins > a.spin_limit) { __hip_atomic_store(a.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); return; }
                    if ((spins & 127u) == 0 && __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) return;
                    __builtin_amdgcn_s_sleep(1);
                    v = __hip_atomic_load(wd + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                lds[i & 4095] = __uint_as_float((unsigned)v);
            }
            __syncthreads();
        } else {
            float *b = a.buf + ((long long)(it & 1) * a.n_teams + team) * a.len;
            for (int i = lo + threadIdx.x; i < hi; i += kT)
                __hip_atomic_store(reinterpret_cast<unsigned *>(b + i), (unsigned)(it + i), __ATOMIC_RELAXED,
                                   __HIP_MEMORY_SCOPE_AGENT);
            asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
            __syncthreads();
            if (threadIdx.x == 0) {
                unsigned *ctr = a.ctr + team * 32;
                __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                unsigned spins = 0;
                int ok = 1;
                while (__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < (unsigned)it * a.team_size) {
                    if (++spins > a.spin_limit) { __hip_atomic_store(a.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); ok = 0; break; }
                    if ((spins & 127u) == 0 && __hip_atomic_load(a.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) { ok = 0; break; }
                    __builtin_amdgcn_s_sleep(1);
                }
                ok_s = ok;
            }
            __syncthreads();
            if (!ok_s) return;
            for (int i = threadIdx.x; i < a.len; i += kT)
                lds[i & 4095] = __uint_as_float(__hip_atomic_load(reinterpret_cast<unsigned *>(b + i), __ATOMIC_RELAXED,
                                                                  __HIP_MEMORY_SCOPE_AGENT));
            __syncthreads();
        }
        acc += lds[(threadIdx.x * 7 + it) % (a.len < 4096 ? a.len : 4096)];
        __syncthreads();
    }
    if (threadIdx.x == 0) a.out[blockIdx.x] = acc;
}

// ---- mfma -----------------------------------------------------------------------------------
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

__global__ void __launch_bounds__(kT) mfma_kernel(int iters, int shape, float *sink)
{
    const float a = 1.0f + threadIdx.x * 1e-6f, b = 0.5f;
    float r = 0.f;
    if (shape == 0) {
        v4f acc[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[i] = (v4f){0.f, 0.f, 0.f, 0.f};
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[i] = __builtin_amdgcn_mfma_f32_4x4x1f32(a, b, acc[i], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 8; ++i) r += acc[i][0];
    } else {
        v16f acc[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
        for (int it = 0; it < iters; ++it)
#pragma unroll
            for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 4; ++i) r += acc[i][0];
    }
    if (r == 12345.678f) sink[blockIdx.x] = r;
}

int n_compute_units(int *out)
{
    int dev = 0;
    PROBE_TRY(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    PROBE_TRY(hipGetDeviceProperties(&prop, dev));
    *out = (prop.multiProcessorCount / 32) * 32;
    return *out >= 32 ? RNNT_OK : RNNT_ERR_UNSUPPORTED;
}

struct Timer {
    hipEvent_t a = nullptr, b = nullptr;
    ~Timer() { if (a) (void)hipEventDestroy(a); if (b) (void)hipEventDestroy(b); }
};

}  // namespace

// Every e4m3 code through the conversion the bfloat16 mode with e4m3-stored weights uses, in
// each of the four byte positions of a word: out[pos * 256 + code] = the bf16 it becomes.
__global__ void widen_kernel(float scale, uint16_t *out)
{
    const unsigned code = threadIdx.x;
    for (int pos = 0; pos < 4; ++pos) {
        const unsigned word = code << (8 * pos);
        const unsigned lo = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(word, scale, false));
        const unsigned hi = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(word, scale, true));
        const unsigned two = pos < 2 ? lo : hi;
        out[pos * 256 + code] = (uint16_t)((pos & 1) ? (two >> 16) : (two & 0xffffu));
    }
}

__global__ void widen4_kernel(float scale, uint16_t *out)
{
    const unsigned byte = threadIdx.x;
    unsigned two[4];
    two[0] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(byte, scale, 0));
    two[1] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(byte << 8, scale, 1));
    two[2] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(byte << 16, scale, 2));
    two[3] = __builtin_bit_cast(unsigned, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(byte << 24, scale, 3));
    for (int pos = 0; pos < 4; ++pos) {
        out[(pos * 256 + byte) * 2] = (uint16_t)(two[pos] & 0xffffu);
        out[(pos * 256 + byte) * 2 + 1] = (uint16_t)(two[pos] >> 16);
    }
}

extern "C" {

int rnnt_probe_stream(int32_t from_l2, double *gbytes_per_s_out, double *per_cu_out)
{
    if (!gbytes_per_s_out || !per_cu_out) return RNNT_ERR_NULL;
    int n_wg = 0;
    int rc = n_compute_units(&n_wg);
    if (rc) return rc;
    // L2 case: 16 chunks of 1.5 MiB; chunk c is read by the work-groups i with i % 16 == c, which the
    // round-robin dispatch puts on XCD c % 8, so an XCD keeps 3 MiB in its 4 MiB L2, as in the decode
    // kernel's layout with teams of 16.  HBM case: every work-group has its own 8 MiB, read once per
    // launch, 2 GiB in all.
    const long long chunk_bytes = from_l2 ? (3ll << 19) : (8ll << 20);
    const int n_chunks = from_l2 ? 16 : n_wg;
    const int rounds = from_l2 ? 64 : 1;
    float4 *buf = nullptr;
    float *sink = nullptr;
    PROBE_TRY(hipMalloc(&buf, (size_t)chunk_bytes * n_chunks));
    PROBE_TRY(hipMalloc(&sink, n_wg * sizeof(float)));
    PROBE_TRY(hipMemset(buf, 0, (size_t)chunk_bytes * n_chunks));
    Timer t;
    PROBE_TRY(hipEventCreate(&t.a));
    PROBE_TRY(hipEventCreate(&t.b));
    float best = 1e30f;
    for (int rep = 0; rep < 4; ++rep) {
        PROBE_TRY(hipEventRecord(t.a, nullptr));
        hipLaunchKernelGGL(stream_kernel, dim3(n_wg), dim3(kT), 0, nullptr, buf, chunk_bytes / 16, n_chunks,
                           rounds, sink);
        PROBE_TRY(hipGetLastError());
        PROBE_TRY(hipEventRecord(t.b, nullptr));
        PROBE_TRY(hipEventSynchronize(t.b));
        float ms = 0.f;
        PROBE_TRY(hipEventElapsedTime(&ms, t.a, t.b));
        if (rep) best = std::min(best, ms);       // the first launch warms the L2
    }
    const long long per_wg = (chunk_bytes / (16 * 8 * kT)) * (16 * 8 * kT) * rounds;
    *gbytes_per_s_out = (double)per_wg * n_wg / (best * 1e-3) / 1e9;
    *per_cu_out = *gbytes_per_s_out / n_wg;
    (void)hipFree(buf);
    (void)hipFree(sink);
    return RNNT_OK;
}

int rnnt_probe_exchange(int32_t team_size, int32_t len, int32_t tagged, double *us_per_exchange_out)
{
    if (!us_per_exchange_out) return RNNT_ERR_NULL;
    int n_wg = 0;
    int rc = n_compute_units(&n_wg);
    if (rc) return rc;
    if (team_size < 1 || n_wg % team_size != 0 || len < team_size || len > (1 << 20)) return RNNT_ERR_SHAPE;
    int coop = 0, dev = 0;
    PROBE_TRY(hipGetDevice(&dev));
    PROBE_TRY(hipDeviceGetAttribute(&coop, hipDeviceAttributeCooperativeLaunch, dev));
    if (!coop) return RNNT_ERR_UNSUPPORTED;
    XParams a{};
    a.n_teams = n_wg / team_size; a.team_size = team_size; a.len = len; a.iters = 2000; a.tagged = tagged ? 1 : 0;
    a.spin_limit = 1u << 22;
    PROBE_TRY(hipMalloc(&a.buf, (size_t)2 * a.n_teams * len * sizeof(float)));
    PROBE_TRY(hipMalloc(&a.words, (size_t)2 * a.n_teams * len * sizeof(unsigned long long)));
    PROBE_TRY(hipMalloc(&a.ctr, (size_t)a.n_teams * 32 * sizeof(unsigned)));
    PROBE_TRY(hipMalloc(&a.abort_flag, sizeof(unsigned)));
    PROBE_TRY(hipMalloc(&a.out, n_wg * sizeof(float)));
    Timer t;
    PROBE_TRY(hipEventCreate(&t.a));
    PROBE_TRY(hipEventCreate(&t.b));
    float best = 1e30f;
    unsigned aborted = 0;
    for (int rep = 0; rep < 3; ++rep) {
        PROBE_TRY(hipMemset(a.words, 0, (size_t)2 * a.n_teams * len * sizeof(unsigned long long)));
        PROBE_TRY(hipMemset(a.ctr, 0, (size_t)a.n_teams * 32 * sizeof(unsigned)));
        PROBE_TRY(hipMemset(a.abort_flag, 0, sizeof(unsigned)));
        void *args[] = {&a};
        PROBE_TRY(hipEventRecord(t.a, nullptr));
        PROBE_TRY(hipLaunchCooperativeKernel(reinterpret_cast<const void *>(exchange_kernel), dim3(n_wg), dim3(kT),
                                             args, 0, nullptr));
        PROBE_TRY(hipEventRecord(t.b, nullptr));
        PROBE_TRY(hipEventSynchronize(t.b));
        float ms = 0.f;
        PROBE_TRY(hipEventElapsedTime(&ms, t.a, t.b));
        best = std::min(best, ms);
        PROBE_TRY(hipMemcpy(&aborted, a.abort_flag, sizeof aborted, hipMemcpyDeviceToHost));
        if (aborted) break;
    }
    (void)hipFree(a.buf); (void)hipFree(a.words); (void)hipFree(a.ctr); (void)hipFree(a.abort_flag); (void)hipFree(a.out);
    if (aborted) return rnnt::hip_fail(hipErrorLaunchTimeOut, "exchange probe: a bounded wait expired");
    *us_per_exchange_out = (double)best * 1e3 / a.iters;
    return RNNT_OK;
}

int rnnt_probe_e4m3_widening(float scale, uint16_t *bf16_out)
{
    if (!bf16_out) return RNNT_ERR_NULL;
    uint16_t *dev = nullptr;
    PROBE_TRY(hipMalloc(&dev, 4 * 256 * sizeof(uint16_t)));
    hipLaunchKernelGGL(widen_kernel, dim3(1), dim3(256), 0, nullptr, scale, dev);
    PROBE_TRY(hipGetLastError());
    PROBE_TRY(hipMemcpy(bf16_out, dev, 4 * 256 * sizeof(uint16_t), hipMemcpyDeviceToHost));
    (void)hipFree(dev);
    return RNNT_OK;
}

int rnnt_probe_e2m1_widening(float scale, uint16_t *bf16_out)
{
    if (!bf16_out) return RNNT_ERR_NULL;
    uint16_t *dev = nullptr;
    PROBE_TRY(hipMalloc(&dev, 4 * 256 * 2 * sizeof(uint16_t)));
    hipLaunchKernelGGL(widen4_kernel, dim3(1), dim3(256), 0, nullptr, scale, dev);
    PROBE_TRY(hipGetLastError());
    PROBE_TRY(hipMemcpy(bf16_out, dev, 4 * 256 * 2 * sizeof(uint16_t), hipMemcpyDeviceToHost));
    (void)hipFree(dev);
    return RNNT_OK;
}

int rnnt_probe_mfma(int32_t shape, double *tflops_out)
{
    if (!tflops_out) return RNNT_ERR_NULL;
    if (shape != 0 && shape != 1) return RNNT_ERR_SHAPE;
    int n_wg = 0;
    int rc = n_compute_units(&n_wg);
    if (rc) return rc;
    float *sink = nullptr;
    PROBE_TRY(hipMalloc(&sink, n_wg * sizeof(float)));
    Timer t;
    PROBE_TRY(hipEventCreate(&t.a));
    PROBE_TRY(hipEventCreate(&t.b));
    const int iters = 20000;
    float best = 1e30f;
    for (int rep = 0; rep < 3; ++rep) {
        PROBE_TRY(hipEventRecord(t.a, nullptr));
        hipLaunchKernelGGL(mfma_kernel, dim3(n_wg), dim3(kT), 0, nullptr, iters, shape, sink);
        PROBE_TRY(hipGetLastError());
        PROBE_TRY(hipEventRecord(t.b, nullptr));
        PROBE_TRY(hipEventSynchronize(t.b));
        float ms = 0.f;
        PROBE_TRY(hipEventElapsedTime(&ms, t.a, t.b));
        best = std::min(best, ms);
    }
    (void)hipFree(sink);
    // flops per wave instruction: 4x4x1 in 16 blocks = 512; 32x32x2 = 4096
    const double per_wave = shape == 0 ? 8.0 * 512.0 : 4.0 * 4096.0;
    *tflops_out = per_wave * iters * (kT / 64) * n_wg / (best * 1e-3) / 1e12;
    return RNNT_OK;
}

}  // extern "C"
