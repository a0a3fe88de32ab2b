// Encoder-side joint projection  P[b, t, :] = W_enc x[b, t, :] + b_enc  for every
// valid frame, as one MFMA GEMM (fp32: v_mfma_f32_32x32x2_f32; bfloat16 mode:
// v_mfma_f32_32x32x8_bf16_1k), and the one-time folding of the embedding table into the
// first LSTM layer's input term.
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
template <int BM>
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
                As[kk + 0][r] = ra[i].x; As[kk + 1][r] = ra[i].y;
                As[kk + 2][r] = ra[i].z; As[kk + 3][r] = ra[i].w;
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

// The same product in the bfloat16 mode, on the bf16 matrix cores (v_mfma_f32_32x32x8_bf16_1k):
// the frames are rounded to bfloat16 (ties to even) as they are staged, the engine's copy of
// W_enc holds bfloat16 values already (its low halves are zero), products are exact in fp32 and
// the sums are fp32.  Both operands have K contiguous in memory, which is what the instruction
// wants per lane (four consecutive k of one row), so the tiles sit in LDS row-major as bf16 and
// nothing is transposed.  Same grid and wave arrangement as the fp32 kernel, K tiles of 32.
typedef short v4s_ __attribute__((ext_vector_type(4)));
constexpr int KTB = 32, LDB = KTB + 4;       // bf16 per LDS row: 72 bytes, 8-byte aligned rows

__device__ __forceinline__ uint2 pack_bf16x4_rne(float4 v)
{
    const unsigned a = __float_as_uint(bf16_rne(v.x)) >> 16, b = __float_as_uint(bf16_rne(v.y)) >> 16;
    const unsigned c = __float_as_uint(bf16_rne(v.z)) >> 16, d = __float_as_uint(bf16_rne(v.w)) >> 16;
    return make_uint2(a | (b << 16), c | (d << 16));
}

template <int BM>
__global__ void __launch_bounds__(256)
enc_proj_bf16_kernel(const float *__restrict__ x, const int *__restrict__ enc_len,
                     const float *__restrict__ w_enc, const float *__restrict__ b_enc,
                     float *__restrict__ proj, int T, int F, int J)
{
    constexpr int MI = BM / 64;
    constexpr int NA = BM / 32;          // float4 of A a thread stages per K tile (BM * 8 / 256)
    constexpr int NB = BN / 32;
    __shared__ __align__(16) unsigned short As[BM][LDB];
    __shared__ __align__(16) unsigned short Bs[BN][LDB];
    const int b = blockIdx.z;
    int len = enc_len[b];
    len = min(max(len, 0), T);
    const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
    if (m0 >= len) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const float *xa = x + (long long)b * T * F;
    // float4 number idx of a tile: row idx / 8, k = 4 * (idx % 8)
    const float *a_src[NA], *b_src[NB];
    bool b_ok[NB];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int idx = tid + i * 256;
        a_src[i] = xa + (long long)min(m0 + (idx >> 3), T - 1) * F + (idx & 7) * 4;
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int idx = tid + i * 256, n = n0 + (idx >> 3);
        b_ok[i] = n < J;
        b_src[i] = w_enc + (long long)min(n, J - 1) * F + (idx & 7) * 4;
    }
    v16f acc[MI][2];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
    float4 ra[NA], rb[NB];
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    // K is a multiple of 16 (checked when the engine is created); a last half tile reads zeros
    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            ra[i] = zero4;
            if (k0 + ((tid + i * 256) & 7) * 4 < F) ra[i] = *reinterpret_cast<const float4 *>(a_src[i] + k0);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            rb[i] = zero4;
            if (b_ok[i] && k0 + ((tid + i * 256) & 7) * 4 < F) rb[i] = *reinterpret_cast<const float4 *>(b_src[i] + k0);
        }
    };
    fetch(0);
    const int kh = lane >> 5, c = lane & 31;
    for (int k0 = 0; k0 < F; k0 += KTB) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int idx = tid + i * 256;
            *reinterpret_cast<uint2 *>(&As[idx >> 3][(idx & 7) * 4]) = pack_bf16x4_rne(ra[i]);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int idx = tid + i * 256;
            // the weights are bfloat16 values: their upper halves are the codes
            const uint2 wv = make_uint2((__float_as_uint(rb[i].x) >> 16) | (__float_as_uint(rb[i].y) & 0xffff0000u),
                                        (__float_as_uint(rb[i].z) >> 16) | (__float_as_uint(rb[i].w) & 0xffff0000u));
            *reinterpret_cast<uint2 *>(&Bs[idx >> 3][(idx & 7) * 4]) = wv;
        }
        __syncthreads();
        if (k0 + KTB < F) fetch(k0 + KTB);
#pragma unroll
        for (int ks = 0; ks < KTB / 8; ++ks) {
            const int k = ks * 8 + kh * 4;
            const v4s_ b0 = *reinterpret_cast<const v4s_ *>(&Bs[wn * 64 + c][k]);
            const v4s_ b1 = *reinterpret_cast<const v4s_ *>(&Bs[wn * 64 + 32 + c][k]);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const v4s_ a = *reinterpret_cast<const v4s_ *>(&As[wm * 32 * MI + mi * 32 + c][k]);
                acc[mi][0] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a, b0, acc[mi][0], 0, 0, 0);
                acc[mi][1] = __builtin_amdgcn_mfma_f32_32x32x8bf16_1k(a, b1, acc[mi][1], 0, 0, 0);
            }
        }
    }
    // accumulator register v of lane l holds row 8*(v/4) + 4*(l/32) + v%4, column l%32
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
            hipLaunchKernelGGL((enc_proj_bf16_kernel<64>), grid, dim3(256), 0, stream, enc_out, enc_len, w_enc,
                               b_enc, proj, T, F, J);
        else
            hipLaunchKernelGGL((enc_proj_kernel<64>), grid, dim3(256), 0, stream, enc_out, enc_len, w_enc,
                               b_enc, proj, T, F, J);
    } else {
        if (round_x)
            hipLaunchKernelGGL((enc_proj_bf16_kernel<128>), grid, dim3(256), 0, stream, enc_out, enc_len, w_enc,
                               b_enc, proj, T, F, J);
        else
            hipLaunchKernelGGL((enc_proj_kernel<128>), grid, dim3(256), 0, stream, enc_out, enc_len, w_enc,
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
