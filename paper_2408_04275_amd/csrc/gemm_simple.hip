// General strided GEMM on the vector ALUs with fp32 FMA: the fp32 storage path, and the
// path for bf16 shapes the MFMA kernel does not take (rows not 16-byte aligned).
// 64x64 output tile per 256-thread workgroup, 16-deep K slices staged through LDS, a 4x4
// register block per thread.
#include "kernels.h"

namespace mmt {

constexpr int SB = 64, SK = 16;

template <typename T, typename TC>
__global__ __launch_bounds__(256) void gemm_simple_kernel(int M, int N, int K, const T *__restrict__ A, long sam,
                                                          long sak, const T *__restrict__ B, long sbn, long sbk,
                                                          TC *__restrict__ C, int ldc, const T *__restrict__ bias,
                                                          const T *__restrict__ residual, bool accumulate) {
    __shared__ float As[SK][SB + 4], Bs[SK][SB + 4];
    const int m0 = blockIdx.y * SB, n0 = blockIdx.x * SB;
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += SK) {
        // 64 x 16 elements per operand, 4 per thread.  Consecutive threads walk the
        // operand's contiguous direction.
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int e = threadIdx.x + i * 256;
            int r, k;
            if (sak == 1) { k = e & 15; r = e >> 4; } else { r = e & 63; k = e >> 6; }
            float v = 0.f;
            if (m0 + r < M && k0 + k < K) v = Elem<T>::load(A + (long)(m0 + r) * sam + (long)(k0 + k) * sak);
            As[k][r] = v;
            if (sbk == 1) { k = e & 15; r = e >> 4; } else { r = e & 63; k = e >> 6; }
            v = 0.f;
            if (n0 + r < N && k0 + k < K) v = Elem<T>::load(B + (long)(n0 + r) * sbn + (long)(k0 + k) * sbk);
            Bs[k][r] = v;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < SK; ++k) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            float v = acc[i][j];
            if (bias) v += Elem<T>::load(bias + n);
            if (residual) v += Elem<T>::load(residual + (long)m * ldc + n);
            if (accumulate) v += Elem<TC>::load(C + (long)m * ldc + n);
            Elem<TC>::store(C + (long)m * ldc + n, v);
        }
    }
}

template <typename T, typename TC>
__global__ void gemm_k0_kernel(int M, int N, TC *__restrict__ C, int ldc, const T *__restrict__ bias,
                               const T *__restrict__ residual) {
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)M * N) return;
    const int m = (int)(idx / N), n = (int)(idx % N);
    float v = 0.f;
    if (bias) v += Elem<T>::load(bias + n);
    if (residual) v += Elem<T>::load(residual + (long)m * ldc + n);
    Elem<TC>::store(C + (long)m * ldc + n, v);
}

template <typename T, typename TC>
static hipError_t launch(const GemmArgs &g, hipStream_t st) {
    if (g.M == 0 || g.N == 0) return hipSuccess;
    if (g.K == 0) {                       // empty contraction: C = bias + residual (or unchanged)
        if (g.accumulate) return hipSuccess;
        gemm_k0_kernel<T, TC><<<ceil_div((long)g.M * g.N, 256), 256, 0, st>>>(g.M, g.N, (TC *)g.C, g.ldc, (const T *)g.bias,
                                                                          (const T *)g.residual);
        return hipGetLastError();
    }
    long sam, sak, sbn, sbk;
    if (g.layout == GEMM_TN) { sam = 1; sak = g.lda; } else { sam = g.lda; sak = 1; }
    if (g.layout == GEMM_NT) { sbn = g.ldb; sbk = 1; } else { sbn = 1; sbk = g.ldb; }
    dim3 grid(ceil_div(g.N, SB), ceil_div(g.M, SB));
    gemm_simple_kernel<T, TC><<<grid, 256, 0, st>>>(g.M, g.N, g.K, (const T *)g.A, sam, sak, (const T *)g.B, sbn, sbk,
                                                    (TC *)g.C, g.ldc, (const T *)g.bias, (const T *)g.residual, g.accumulate);
    return hipGetLastError();
}

hipError_t gemm_simple(int dtype, const GemmArgs &g, hipStream_t st) {
    if (dtype == DT_F32) return launch<float, float>(g, st);
    return g.c_f32 ? launch<bf16_t, float>(g, st) : launch<bf16_t, bf16_t>(g, st);
}

}  // namespace mmt
