// Encoder-side joint projection  P[b, t, :] = W_enc x[b, t, :] + b_enc  for every
// valid frame, as one fp32 MFMA GEMM (v_mfma_f32_32x32x2_f32), and the one-time
// folding of the embedding table into the first LSTM layer's input term.
#include "engine.h"

namespace rnnt {

typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int BN = 128, KT = 16, LDP = 4;

// nearest bfloat16 value (ties to even) of a float, as a float; NaN and infinities pass through
__device__ __forceinline__ float bf16_rne(float v)
{
    unsigned u = __float_as_uint(v);
    if ((u & 0x7f800000u) != 0x7f800000u) { u += 0x7fffu + ((u >> 16) & 1u); u &= 0xffff0000u; }
    return __uint_as_float(u);
}

// grid: (ceil(T/BM), ceil(J/BN), B); 256 threads = 4 waves in 2 x 2, each a (BM/2) x 64 tile.
// BM = 128 reuses a loaded weight tile for twice the rows; BM = 64 wastes less on the tiles of an
// utterance's last frames and spreads a small batch more evenly over the compute units (the
// launcher picks: 0.228 -> 0.208 ms at B = 32, 0.088 -> 0.055 ms at B = 1, but 0.69 -> 0.74 ms at
// B = 128 with the smaller tile).
// Tiles that start at or beyond enc_len[b] do nothing; rows at t >= enc_len[b]
// inside a tile are computed and not stored.
// ROUND_X: bfloat16 mode, the frames are rounded to bfloat16 as they enter the product (the
// engine's copy of W_enc has been rounded once); products of two such values are exact in fp32.
template <bool ROUND_X, int BM>
__global__ void __launch_bounds__(256)
enc_proj_kernel(const float *__restrict__ x, const int *__restrict__ enc_len,
                const float *__restrict__ w_enc, const float *__restrict__ b_enc,
                float *__restrict__ proj, int T, int F, int J)
{
    constexpr int MI = BM / 64;     // 32-row MFMA tiles of a wave along M (its share of BM is 32 * MI rows)
    __shared__ float As[KT][BM + LDP];
    __shared__ float Bs[KT][BN + LDP];
    const int b = blockIdx.z;
    int len = enc_len[b];
    len = min(max(len, 0), T);
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
    if (m0 >= len) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const float *xa = x + (long long)b * T * F;

    // per K tile a thread moves NA float4 of A and two of B
    constexpr int NA = BM / 64;
    int a_row[2], a_k4[2];
    const float *a_src[NA], *b_src[2];
    bool b_ok[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int idx = tid + i * 256;
        a_row[i] = idx >> 2;
        a_k4[i] = idx & 3;
        if (i < NA) {
            const int t = min(m0 + a_row[i], T - 1);
            a_src[i] = xa + (long long)t * F + a_k4[i] * 4;
        }
        const int n = n0 + a_row[i];
        b_ok[i] = n < J;
        b_src[i] = w_enc + (long long)min(n, J - 1) * F + a_k4[i] * 4;
    }
    v16f acc[MI][2];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

    float4 ra[NA], rb[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        if (i < NA) ra[i] = *reinterpret_cast<const float4 *>(a_src[i]);
        rb[i] = b_ok[i] ? *reinterpret_cast<const float4 *>(b_src[i]) : make_float4(0, 0, 0, 0);
    }
    for (int k0 = 0; k0 < F; k0 += KT) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int kk = a_k4[i] * 4, r = a_row[i];
            if (i < NA) {
                if (ROUND_X) {
                    As[kk + 0][r] = bf16_rne(ra[i].x); As[kk + 1][r] = bf16_rne(ra[i].y);
                    As[kk + 2][r] = bf16_rne(ra[i].z); As[kk + 3][r] = bf16_rne(ra[i].w);
                } else {
                    As[kk + 0][r] = ra[i].x; As[kk + 1][r] = ra[i].y;
                    As[kk + 2][r] = ra[i].z; As[kk + 3][r] = ra[i].w;
                }
            }
            Bs[kk + 0][r] = rb[i].x; Bs[kk + 1][r] = rb[i].y;
            Bs[kk + 2][r] = rb[i].z; Bs[kk + 3][r] = rb[i].w;
        }
        __syncthreads();
        if (k0 + KT < F) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                if (i < NA) ra[i] = *reinterpret_cast<const float4 *>(a_src[i] + k0 + KT);
                rb[i] = b_ok[i] ? *reinterpret_cast<const float4 *>(b_src[i] + k0 + KT)
                                : make_float4(0, 0, 0, 0);
            }
        }
        const int kh = lane >> 5, c = lane & 31;
#pragma unroll
        for (int kk = 0; kk < KT; kk += 2) {
            const float b0 = Bs[kk + kh][wn * 64 + c];
            const float b1 = Bs[kk + kh][wn * 64 + 32 + c];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const float a = As[kk + kh][wm * 32 * MI + mi * 32 + c];
                acc[mi][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b0, acc[mi][0], 0, 0, 0);
                acc[mi][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b1, acc[mi][1], 0, 0, 0);
            }
        }
    }
    // accumulator register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32
    const int kh = lane >> 5, c = lane & 31;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            const int col = n0 + wn * 64 + ni * 32 + c;
            if (col >= J) continue;
            const float bias = b_enc[col];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm * 32 * MI + mi * 32 + 8 * (v >> 2) + 4 * kh + (v & 3);
                if (row < len) proj[((long long)b * T + row) * J + col] = acc[mi][ni][v] + bias;
            }
        }
}

hipError_t launch_encoder_projection(const float *enc_out, const int *enc_len, const float *w_enc,
                                     const float *b_enc, float *proj, int B, int T, int F, int J,
                                     bool round_x, hipStream_t stream)
{
    // the smaller row tile while the larger one would give each compute unit only a few blocks
    const long long blocks128 = (long long)((T + 127) / 128) * ((J + BN - 1) / BN) * B;
    const bool small_tile = blocks128 <= 1024;
    const int bm = small_tile ? 64 : 128;
    const dim3 grid((T + bm - 1) / bm, (J + BN - 1) / BN, B);
    if (small_tile) {
        if (round_x)
            hipLaunchKernelGGL((enc_proj_kernel<true, 64>), grid, dim3(256), 0, stream, enc_out, enc_len, w_enc,
                               b_enc, proj, T, F, J);
        else
            hipLaunchKernelGGL((enc_proj_kernel<false, 64>), grid, dim3(256), 0, stream, enc_out, enc_len, w_enc,
                               b_enc, proj, T, F, J);
    } else {
        if (round_x)
            hipLaunchKernelGGL((enc_proj_kernel<true, 128>), grid, dim3(256), 0, stream, enc_out, enc_len, w_enc,
                               b_enc, proj, T, F, J);
        else
            hipLaunchKernelGGL((enc_proj_kernel<false, 128>), grid, dim3(256), 0, stream, enc_out, enc_len, w_enc,
                               b_enc, proj, T, F, J);
    }
    return hipGetLastError();
}

__global__ void round_bf16_kernel(float *v, long long n)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) v[i] = bf16_rne(v[i]);
}

hipError_t launch_round_bf16(float *v, long long n, hipStream_t stream)
{
    hipLaunchKernelGGL(round_bf16_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, v, n);
    return hipGetLastError();
}

// one thread per (label v, unit u, gate g)
__global__ void fold_embedding_kernel(const float *__restrict__ emb, const float *__restrict__ w_ih0,
                                      const float *__restrict__ b_ih0,
                                      const float *__restrict__ b_hh0, float *__restrict__ T0, int V1,
                                      int E, int H, int round_bf16)
{
    const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long long)V1 * H * 4) return;
    const int g = (int)(idx & 3);
    const int u = (int)((idx >> 2) % H);
    const int v = (int)((idx >> 2) / H);
    const float *wr = w_ih0 + (long long)(g * H + u) * E;
    const float *er = emb + (long long)v * E;
    float s = 0.f;
    if (round_bf16) { for (int e = 0; e < E; ++e) s += bf16_rne(wr[e]) * bf16_rne(er[e]); }
    else { for (int e = 0; e < E; ++e) s += wr[e] * er[e]; }
    T0[idx] = s + b_ih0[g * H + u] + b_hh0[g * H + u];
}

hipError_t launch_fold_embedding(const float *emb, const float *w_ih0, const float *b_ih0,
                                 const float *b_hh0, float *T0, int V1, int E, int H,
                                 bool round_bf16, hipStream_t stream)
{
    const long long n = (long long)V1 * H * 4;
    hipLaunchKernelGGL(fold_embedding_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream,
                       emb, w_ih0, b_ih0, b_hh0, T0, V1, E, H, round_bf16 ? 1 : 0);
    return hipGetLastError();
}

}  // namespace rnnt
