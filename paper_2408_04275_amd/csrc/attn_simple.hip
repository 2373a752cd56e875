// Segment-masked attention on the vector ALUs, fp32 arithmetic: the fp32 storage path.
// One wavefront owns one (token, head); the head dimension is spread over the 64 lanes and
// keys are visited one by one with an online softmax.  Masking is by construction: the key
// loop runs over exactly the allowed keys of the token's own segment.
#include "kernels.h"

namespace mmt {

template <typename T, int E>
__device__ __forceinline__ void load_row(const T *p, int lane, float (&v)[E]) {
#pragma unroll
    for (int e = 0; e < E; ++e) v[e] = Elem<T>::load(p + lane + 64 * e);
}

template <typename T, int E>
__global__ __launch_bounds__(256) void attn_simple_fwd_kernel(AttnArgs a) {
    const int lane = threadIdx.x & 63;
    const long w = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= (long)a.T * a.nh) return;
    const int h = (int)(w / a.T), i = (int)(w % a.T);
    const int g = h / (a.nh / a.nkv);
    const int seg = a.tok_seg[i];
    const int s0 = a.cu[seg], s1 = a.cu[seg + 1];
    const int mode = a.modes ? a.modes[seg] : a.default_mode;
    const int jend = mode == MASK_CAUSAL ? i + 1 : s1;
    const T *base = (const T *)a.qkv;
    const int nq = a.nh * a.d, nk = a.nkv * a.d;
    float q[E], acc[E], k[E], v[E];
    load_row<T, E>(base + (long)i * a.ld_qkv + h * a.d, lane, q);
#pragma unroll
    for (int e = 0; e < E; ++e) acc[e] = 0.f;
    float m = -INFINITY, l = 0.f;
    for (int j = s0; j < jend; ++j) {
        load_row<T, E>(base + (long)j * a.ld_qkv + nq + g * a.d, lane, k);
        load_row<T, E>(base + (long)j * a.ld_qkv + nq + nk + g * a.d, lane, v);
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) s += q[e] * k[e];
        s = wave_sum(s) * a.scale;
        const float mn = fmaxf(m, s);
        const float corr = expf(m - mn), p = expf(s - mn);
        l = l * corr + p;
#pragma unroll
        for (int e = 0; e < E; ++e) acc[e] = acc[e] * corr + p * v[e];
        m = mn;
    }
    T *o = (T *)a.o + (long)i * nq + h * a.d;
#pragma unroll
    for (int e = 0; e < E; ++e) Elem<T>::store(o + lane + 64 * e, acc[e] / l);
    if (lane == 0) a.lse[(long)h * a.T + i] = m + logf(l);
}

// dQ_i = scale * sum_j dS_ij k_j,  dS_ij = P_ij (dO_i . v_j - D_i),  D_i = dO_i . O_i,  P_ij = exp(s_ij - lse_i)
template <typename T, int E>
__global__ __launch_bounds__(256) void attn_simple_dq_kernel(AttnArgs a) {
    const int lane = threadIdx.x & 63;
    const long w = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= (long)a.T * a.nh) return;
    const int h = (int)(w / a.T), i = (int)(w % a.T);
    const int g = h / (a.nh / a.nkv);
    const int seg = a.tok_seg[i];
    const int s0 = a.cu[seg], s1 = a.cu[seg + 1];
    const int mode = a.modes ? a.modes[seg] : a.default_mode;
    const int jend = mode == MASK_CAUSAL ? i + 1 : s1;
    const T *base = (const T *)a.qkv;
    const int nq = a.nh * a.d, nk = a.nkv * a.d;
    float q[E], dO[E], O[E], dq[E], k[E], v[E];
    load_row<T, E>(base + (long)i * a.ld_qkv + h * a.d, lane, q);
    load_row<T, E>((const T *)a.d_o + (long)i * nq + h * a.d, lane, dO);
    load_row<T, E>((const T *)a.o + (long)i * nq + h * a.d, lane, O);
    float D = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) { D += dO[e] * O[e]; dq[e] = 0.f; }
    D = wave_sum(D);
    if (lane == 0) a.Dsum[(long)h * a.T + i] = D;
    const float lse = a.lse[(long)h * a.T + i];
    for (int j = s0; j < jend; ++j) {
        load_row<T, E>(base + (long)j * a.ld_qkv + nq + g * a.d, lane, k);
        load_row<T, E>(base + (long)j * a.ld_qkv + nq + nk + g * a.d, lane, v);
        float s = 0.f, dp = 0.f;
#pragma unroll
        for (int e = 0; e < E; ++e) { s += q[e] * k[e]; dp += dO[e] * v[e]; }
        s = wave_sum(s) * a.scale;
        dp = wave_sum(dp);
        const float ds = expf(s - lse) * (dp - D);
#pragma unroll
        for (int e = 0; e < E; ++e) dq[e] += ds * k[e];
    }
    T *out = (T *)a.d_qkv + (long)i * a.ld_qkv + h * a.d;
#pragma unroll
    for (int e = 0; e < E; ++e) Elem<T>::store(out + lane + 64 * e, dq[e] * a.scale);
}

// dK_j = scale * sum_{h in group} sum_i dS_ij q_i,   dV_j = sum_{h in group} sum_i P_ij dO_i
template <typename T, int E>
__global__ __launch_bounds__(256) void attn_simple_dkv_kernel(AttnArgs a) {
    const int lane = threadIdx.x & 63;
    const long w = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (w >= (long)a.T * a.nkv) return;
    const int g = (int)(w / a.T), j = (int)(w % a.T);
    const int group = a.nh / a.nkv;
    const int seg = a.tok_seg[j];
    const int s0 = a.cu[seg], s1 = a.cu[seg + 1];
    const int mode = a.modes ? a.modes[seg] : a.default_mode;
    const int ibeg = mode == MASK_CAUSAL ? j : s0;
    const T *base = (const T *)a.qkv;
    const int nq = a.nh * a.d, nk = a.nkv * a.d;
    float k[E], v[E], dk[E], dv[E], q[E], dO[E];
    load_row<T, E>(base + (long)j * a.ld_qkv + nq + g * a.d, lane, k);
    load_row<T, E>(base + (long)j * a.ld_qkv + nq + nk + g * a.d, lane, v);
#pragma unroll
    for (int e = 0; e < E; ++e) { dk[e] = 0.f; dv[e] = 0.f; }
    for (int h = g * group; h < (g + 1) * group; ++h) {
        for (int i = ibeg; i < s1; ++i) {
            load_row<T, E>(base + (long)i * a.ld_qkv + h * a.d, lane, q);
            load_row<T, E>((const T *)a.d_o + (long)i * nq + h * a.d, lane, dO);
            float s = 0.f, dp = 0.f;
#pragma unroll
            for (int e = 0; e < E; ++e) { s += q[e] * k[e]; dp += dO[e] * v[e]; }
            s = wave_sum(s) * a.scale;
            dp = wave_sum(dp);
            const float p = expf(s - a.lse[(long)h * a.T + i]);
            const float ds = p * (dp - a.Dsum[(long)h * a.T + i]);
#pragma unroll
            for (int e = 0; e < E; ++e) { dv[e] += p * dO[e]; dk[e] += ds * q[e]; }
        }
    }
    T *okp = (T *)a.d_qkv + (long)j * a.ld_qkv + nq + g * a.d;
    T *ovp = (T *)a.d_qkv + (long)j * a.ld_qkv + nq + nk + g * a.d;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        Elem<T>::store(okp + lane + 64 * e, dk[e] * a.scale);
        Elem<T>::store(ovp + lane + 64 * e, dv[e]);
    }
}

hipError_t attn_simple_fwd(int dtype, const AttnArgs &a, hipStream_t st) {
    if (a.T == 0) return hipSuccess;
    const int grid = ceil_div((long)a.T * a.nh, 4);
#define L(TT, EE) attn_simple_fwd_kernel<TT, EE><<<grid, 256, 0, st>>>(a)
    if (dtype == DT_F32) { if (a.d == 64) L(float, 1); else L(float, 2); }
    else { if (a.d == 64) L(bf16_t, 1); else L(bf16_t, 2); }
#undef L
    return hipGetLastError();
}

hipError_t attn_simple_bwd(int dtype, const AttnArgs &a, hipStream_t st) {
    if (a.T == 0) return hipSuccess;
    const int gq = ceil_div((long)a.T * a.nh, 4), gk = ceil_div((long)a.T * a.nkv, 4);
#define L(TT, EE) attn_simple_dq_kernel<TT, EE><<<gq, 256, 0, st>>>(a); attn_simple_dkv_kernel<TT, EE><<<gk, 256, 0, st>>>(a)
    if (dtype == DT_F32) { if (a.d == 64) { L(float, 1); } else { L(float, 2); } }
    else { if (a.d == 64) { L(bf16_t, 1); } else { L(bf16_t, 2); } }
#undef L
    return hipGetLastError();
}

}  // namespace mmt
