// Optimizer step of mixed-precision training on one rank's shard of the parameters (ZeRO-1 gives every
// data-parallel rank 1/DP of the optimizer state): fp32 master weights and Adam moments, fp32 accumulated
// gradients, bf16 (or fp32) working copy of the weights written in the same pass.  Decoupled weight decay
// (AdamW).  Memory-bound: per element it reads 16 bytes and writes 12 + the working copy (+ 4 when the
// gradient is cleared for the next accumulation), 16 bytes per lane per access.
#include "kernels.h"

namespace mmt {

template <typename TP>
__global__ __launch_bounds__(256) void adam_kernel(size_t n, float *__restrict__ w, float *__restrict__ g,
                                                   float *__restrict__ m, float *__restrict__ v, TP *__restrict__ p,
                                                   AdamArgs a) {
    const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= n) return;
    if (i + 4 <= n) {
        f32x4 wv = *reinterpret_cast<const f32x4 *>(w + i), gv = *reinterpret_cast<const f32x4 *>(g + i);
        f32x4 mv = *reinterpret_cast<const f32x4 *>(m + i), vv = *reinterpret_cast<const f32x4 *>(v + i);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float gr = gv[e] * a.grad_scale;
            mv[e] = a.beta1 * mv[e] + a.omb1 * gr;
            vv[e] = a.beta2 * vv[e] + a.omb2 * gr * gr;
            const float upd = (mv[e] * a.inv_bias1) / (sqrtf(vv[e] * a.inv_bias2) + a.eps) + a.weight_decay * wv[e];
            wv[e] -= a.lr * upd;
        }
        *reinterpret_cast<f32x4 *>(w + i) = wv;
        *reinterpret_cast<f32x4 *>(m + i) = mv;
        *reinterpret_cast<f32x4 *>(v + i) = vv;
        if (a.zero_grad) *reinterpret_cast<f32x4 *>(g + i) = f32x4{0.f, 0.f, 0.f, 0.f};
        if (p) {
#pragma unroll
            for (int e = 0; e < 4; ++e) Elem<TP>::store(p + i + e, wv[e]);
        }
    } else {
        for (size_t j = i; j < n; ++j) {
            const float gr = g[j] * a.grad_scale;
            const float mj = a.beta1 * m[j] + a.omb1 * gr;
            const float vj = a.beta2 * v[j] + a.omb2 * gr * gr;
            const float upd = (mj * a.inv_bias1) / (sqrtf(vj * a.inv_bias2) + a.eps) + a.weight_decay * w[j];
            const float wj = w[j] - a.lr * upd;
            w[j] = wj; m[j] = mj; v[j] = vj;
            if (a.zero_grad) g[j] = 0.f;
            if (p) Elem<TP>::store(p + j, wj);
        }
    }
}

hipError_t adam_step(int param_dtype, size_t n, float *w, float *g, float *m, float *v, void *p, const AdamArgs &a,
                     hipStream_t st) {
    if (n == 0) return hipSuccess;
    const size_t blocks = (n + 1023) / 1024;
    if (param_dtype == DT_F32) adam_kernel<float><<<(unsigned)blocks, 256, 0, st>>>(n, w, g, m, v, (float *)p, a);
    else adam_kernel<bf16_t><<<(unsigned)blocks, 256, 0, st>>>(n, w, g, m, v, (bf16_t *)p, a);
    return hipGetLastError();
}

}  // namespace mmt
