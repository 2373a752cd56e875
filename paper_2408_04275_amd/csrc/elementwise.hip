// HBM-bound kernels of the layer: token bookkeeping, RMSNorm / LayerNorm forward and
// backward, rotary embedding, SwiGLU / GELU, column sums.  All arithmetic is fp32;
// storage is fp32 or bf16.  Every kernel moves 16 bytes per lane per access and
// touches each tensor once (rows are re-read from cache, not from HBM).
#include "kernels.h"
#include <atomic>

namespace mmt {

// ---- 8-element vector access --------------------------------------------------------
__device__ __forceinline__ void load8(const float *p, float (&v)[8]) {
    const float4 a = *reinterpret_cast<const float4 *>(p), b = *reinterpret_cast<const float4 *>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t *p, float (&v)[8]) {
    const uint4 a = *reinterpret_cast<const uint4 *>(p);
    const uint32_t w[4] = {a.x, a.y, a.z, a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ void store8(float *p, const float (&v)[8]) {
    *reinterpret_cast<float4 *>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4 *>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(bf16_t *p, const float (&v)[8]) {
    uint4 a;
    a.x = pack_bf16x2(v[0], v[1]); a.y = pack_bf16x2(v[2], v[3]);
    a.z = pack_bf16x2(v[4], v[5]); a.w = pack_bf16x2(v[6], v[7]);
    *reinterpret_cast<uint4 *>(p) = a;
}

// Streaming forms for tensors that a kernel passes over once and that are far larger than the caches.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;
__device__ __forceinline__ void load8_stream(const bf16_t *p, float (&v)[8]) {
    const u32x4_t a = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(a[i] << 16);
        v[2 * i + 1] = __uint_as_float(a[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ void load8_stream(const float *p, float (&v)[8]) { load8(p, v); }
__device__ __forceinline__ void store8_stream(bf16_t *p, const float (&v)[8]) {
    u32x4_t a;
    a[0] = pack_bf16x2(v[0], v[1]); a[1] = pack_bf16x2(v[2], v[3]);
    a[2] = pack_bf16x2(v[4], v[5]); a[3] = pack_bf16x2(v[6], v[7]);
    __builtin_nontemporal_store(a, reinterpret_cast<u32x4_t *>(p));
}
__device__ __forceinline__ void store8_stream(float *p, const float (&v)[8]) { store8(p, v); }

// Eight elements as loaded, not yet widened to fp32: what a kernel holds for a row it has requested ahead of time
// (four registers per chunk in bf16 instead of eight).
template <typename T> struct Raw8;
template <> struct Raw8<bf16_t> { uint4 a; };
template <> struct Raw8<float> { float4 a, b; };
__device__ __forceinline__ void load_raw8(const bf16_t *p, Raw8<bf16_t> &r) {
    // streaming form: each of these tensors is passed over once (norm backward at the 7B shape: 49.8 -> 46.4 us)
    const u32x4_t a = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
    r.a = make_uint4(a[0], a[1], a[2], a[3]);
}
__device__ __forceinline__ void load_raw8(const float *p, Raw8<float> &r) {
    r.a = *reinterpret_cast<const float4 *>(p); r.b = *reinterpret_cast<const float4 *>(p + 4);
}
__device__ __forceinline__ void unpack8(const Raw8<bf16_t> &r, float (&v)[8]) {
    const uint32_t w[4] = {r.a.x, r.a.y, r.a.z, r.a.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[2 * i] = __uint_as_float(w[i] << 16);
        v[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ void unpack8(const Raw8<float> &r, float (&v)[8]) {
    v[0] = r.a.x; v[1] = r.a.y; v[2] = r.a.z; v[3] = r.a.w; v[4] = r.b.x; v[5] = r.b.y; v[6] = r.b.z; v[7] = r.b.w;
}

// ---- token bookkeeping ---------------------------------------------------------------
// tok_seg[t] = s with cu[s] <= t < cu[s+1].
__device__ __forceinline__ int find_segment(const int *__restrict__ cu, int S, int t) {
    int lo = 0, hi = S;               // last s in [0, S) with cu[s] <= t
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (cu[mid] <= t) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ void tok_seg_kernel(const int *__restrict__ cu, const uint8_t *__restrict__ modes, int default_mode,
                               int S, int T, int *__restrict__ tok_seg, int2 *__restrict__ tok_info) {
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= T) return;
    const int s = find_segment(cu, S, t);
    tok_seg[t] = s;
    const int mode = modes ? modes[s] : default_mode;
    tok_info[t] = make_int2(cu[s], cu[s + 1] | (mode == MASK_BIDIR ? (1 << 30) : 0));
}

// rope_cs[t, i] = (cos, sin)(pos(t) * base^(-2i/d)), pos(t) = t - cu[seg(t)]; evaluated in double
// so that the fp32 table is correctly rounded for any position.
__global__ void rope_table_kernel(const int *__restrict__ cu, int S, int T, int d, float rope_base,
                                  float2 *__restrict__ rope_cs) {
    const int half = d >> 1;
    const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (long)T * half) return;
    const int t = (int)(idx / half), i = (int)(idx % half);
    const double pos = (double)(t - cu[find_segment(cu, S, t)]);
    const double phi = pos * exp(-2.0 * i / d * log((double)rope_base));
    rope_cs[idx] = make_float2((float)cos(phi), (float)sin(phi));
}

hipError_t prep_tokens(const int *cu, const uint8_t *modes, int default_mode, int S, int T, int *tok_seg,
                       int2 *tok_info, int d, float rope_base, float2 *rope_cs, hipStream_t st) {
    if (T == 0) return hipSuccess;
    tok_seg_kernel<<<ceil_div(T, 256), 256, 0, st>>>(cu, modes, default_mode, S, T, tok_seg, tok_info);
    if (rope_cs) rope_table_kernel<<<ceil_div((long)T * (d / 2), 256), 256, 0, st>>>(cu, S, T, d, rope_base, rope_cs);
    return hipGetLastError();
}

// ---- normalisation forward -----------------------------------------------------------
// One workgroup per row.  RMSNorm: out = x * rsqrt(mean(x^2) + eps) * g.
// LayerNorm: out = (x - mean) * rsqrt(var_biased + eps) * g + b (variance about the mean, two passes).
template <typename T, bool LN>
__global__ __launch_bounds__(256) void norm_fwd_kernel(const T *__restrict__ x, const T *__restrict__ g,
                                                       const T *__restrict__ b, T *__restrict__ out,
                                                       float *__restrict__ mean, float *__restrict__ rstd,
                                                       int H, float eps) {
    __shared__ float red[4];
    const size_t row = blockIdx.x;
    const T *xr = x + row * H;
    float v[8];
    float mu = 0.f;
    if (LN) {
        float s = 0.f;
        for (int c = threadIdx.x * 8; c < H; c += 2048) {
            load8(xr + c, v);
#pragma unroll
            for (int j = 0; j < 8; ++j) s += v[j];
        }
        mu = block_sum<4>(s, red) / H;
    }
    float ss = 0.f;
    for (int c = threadIdx.x * 8; c < H; c += 2048) {
        load8(xr + c, v);
#pragma unroll
        for (int j = 0; j < 8; ++j) ss += (v[j] - mu) * (v[j] - mu);
    }
    const float r = 1.0f / sqrtf(block_sum<4>(ss, red) / H + eps);
    if (threadIdx.x == 0) {
        rstd[row] = r;
        if (LN) mean[row] = mu;
    }
    float gv[8], bv[8];
    for (int c = threadIdx.x * 8; c < H; c += 2048) {
        load8(xr + c, v);
        load8(g + c, gv);
        if (LN) load8(b + c, bv);
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = (v[j] - mu) * r * gv[j] + (LN ? bv[j] : 0.f);
        store8(out + row * H + c, v);
    }
}

// The same for rows of at most 256 * 8 * MAXC elements, a workgroup walking rows blockIdx.x, blockIdx.x + gridDim.x, ...:
// the row stays in registers between the statistics and the scaling (one read of x), the gain and bias are fetched once
// per workgroup, and the next row is requested before the current one is reduced, so that a workgroup always has a
// row in flight (with one short-lived workgroup per row the kernel reached 5.5 TB/s).
template <typename T, bool LN, int MAXC>
__global__ __launch_bounds__(256) void norm_fwd_rows_kernel(const T *__restrict__ x, const T *__restrict__ g,
                                                            const T *__restrict__ b, T *__restrict__ out,
                                                            float *__restrict__ mean, float *__restrict__ rstd,
                                                            int nrows, int H, float eps) {
    __shared__ float red[4];
    float gv[MAXC][8], bv[LN ? MAXC : 1][8], cur[MAXC][8], nxt[MAXC][8];
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
        const int c = (threadIdx.x + i * 256) * 8;
        if (c < H) {
            load8(g + c, gv[i]);
            if (LN) load8(b + c, bv[i]);
            if (blockIdx.x < nrows) load8(x + (size_t)blockIdx.x * H + c, cur[i]);
        }
    }
    for (size_t row = blockIdx.x; row < (size_t)nrows; row += gridDim.x) {
        const size_t next = row + gridDim.x;
#pragma unroll
        for (int i = 0; i < MAXC; ++i) {
            const int c = (threadIdx.x + i * 256) * 8;
            if (c < H && next < (size_t)nrows) load8(x + next * H + c, nxt[i]);
        }
        float mu = 0.f;
        if (LN) {
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < MAXC; ++i)
                if ((threadIdx.x + i * 256) * 8 < H) {
#pragma unroll
                    for (int j = 0; j < 8; ++j) s += cur[i][j];
                }
            mu = block_sum<4>(s, red) / H;
        }
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < MAXC; ++i)
            if ((threadIdx.x + i * 256) * 8 < H) {
#pragma unroll
                for (int j = 0; j < 8; ++j) ss += (cur[i][j] - mu) * (cur[i][j] - mu);
            }
        const float r = 1.0f / sqrtf(block_sum<4>(ss, red) / H + eps);
        if (threadIdx.x == 0) {
            rstd[row] = r;
            if (LN) mean[row] = mu;
        }
#pragma unroll
        for (int i = 0; i < MAXC; ++i) {
            const int c = (threadIdx.x + i * 256) * 8;
            if (c < H) {
#pragma unroll
                for (int j = 0; j < 8; ++j) cur[i][j] = (cur[i][j] - mu) * r * gv[i][j] + (LN ? bv[i][j] : 0.f);
                store8(out + row * H + c, cur[i]);
#pragma unroll
                for (int j = 0; j < 8; ++j) cur[i][j] = nxt[i][j];
            }
        }
    }
}

// One launch of norm_fwd_rows_kernel: exactly as many workgroups as the device keeps resident at once (a grid one
// workgroup per compute unit larger runs a second, nearly empty round: 22.9 -> 26.9 us at the 7B shape).
template <typename T, bool LN, int MAXC>
hipError_t launch_norm_fwd_rows(const void *x, const void *g, const void *b, void *out, float *mean, float *rstd, int nrows,
                                int H, float eps, hipStream_t st) {
    static std::atomic<int> resident{0};
    int grid = resident.load(std::memory_order_relaxed);
    if (grid == 0) {
        int dev = 0, cus = 0, per_cu = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, norm_fwd_rows_kernel<T, LN, MAXC>, 256, 0);
        if (e != hipSuccess) return e;
        grid = (cus > 0 ? cus : 256) * (per_cu > 0 ? per_cu : 4);
        resident.store(grid, std::memory_order_relaxed);
    }
    if (nrows < grid) grid = nrows;
    norm_fwd_rows_kernel<T, LN, MAXC><<<grid, 256, 0, st>>>((const T *)x, (const T *)g, (const T *)b, (T *)out, mean, rstd, nrows, H, eps);
    return hipGetLastError();
}

hipError_t norm_fwd(int dtype, bool layernorm, const void *x, const void *g, const void *b, void *out,
                    float *mean, float *rstd, int T, int H, float eps, hipStream_t st) {
    if (T == 0) return hipSuccess;
#define R(TT, LNV, MC) return launch_norm_fwd_rows<TT, LNV, MC>(x, g, b, out, mean, rstd, T, H, eps, st)
#define L(TT, LNV) do { if (H % 8 == 0 && H <= 2048) R(TT, LNV, 1); else if (H % 8 == 0 && H <= 4096) R(TT, LNV, 2); else if (H % 8 == 0 && H <= 8192) R(TT, LNV, 4); \
                        else norm_fwd_kernel<TT, LNV><<<T, 256, 0, st>>>((const TT *)x, (const TT *)g, (const TT *)b, (TT *)out, mean, rstd, H, eps); } while (0)
    if (dtype == DT_F32) { if (layernorm) L(float, true); else L(float, false); }
    else { if (layernorm) L(bf16_t, true); else L(bf16_t, false); }
#undef L
#undef R
    return hipGetLastError();
}

// ---- normalisation backward ----------------------------------------------------------
// With xhat = (x - mean) * r and ghat = d_out * g:
//   d_in = r * (ghat - mean_H(ghat) [LayerNorm only] - xhat * mean_H(ghat * xhat)) + d_res
//   dg = sum_t d_out * xhat,  db = sum_t d_out.
// A workgroup walks rows blockIdx.x, blockIdx.x + gridDim.x, ...; each thread owns the same
// columns in every row, so the gain/bias partial sums stay in registers and are written once
// per workgroup to part_g / part_b [gridDim.x, H].
constexpr int NORM_BWD_MAXC = 4;          // column chunks of 8 per thread: H <= 256 * 8 * 4 = 8192 (the kernel is also
                                          // built for 1 and 2 chunks: fewer registers per thread, more rows in flight)
constexpr int NORM_BWD_GRID = 512;

// narrow rows leave registers for more resident workgroups: twice the grid
int norm_bwd_blocks(int T, int H) {
    const int grid = H <= 4096 ? 2 * NORM_BWD_GRID : NORM_BWD_GRID;
    return T < grid ? (T > 0 ? T : 1) : grid;
}

template <typename T, bool LN, int NORM_BWD_MAXC, bool COLS>
__global__ __launch_bounds__(256) void norm_bwd_kernel(const T *__restrict__ d_out, const T *__restrict__ x,
                                                       const T *__restrict__ g, const float *__restrict__ mean,
                                                       const float *__restrict__ rstd, const T *__restrict__ d_res,
                                                       T *__restrict__ d_in, float *__restrict__ part_g,
                                                       float *__restrict__ part_b, float *__restrict__ part_din,
                                                       float *__restrict__ part_dres, int nrows, int H) {
    __shared__ float red[4];
    float gv[NORM_BWD_MAXC][8], ag[NORM_BWD_MAXC][8], ab[NORM_BWD_MAXC][8];
    // COLS: column sums of the result and of the added gradient as well (the bias gradients of the two linears
    // that sit on either side of the normalisation's residual branch)
    float ad[COLS ? NORM_BWD_MAXC : 1][8], ae[COLS ? NORM_BWD_MAXC : 1][8];
#pragma unroll
    for (int i = 0; i < NORM_BWD_MAXC; ++i) {
        const int c = (threadIdx.x + i * 256) * 8;
        if (c < H) load8(g + c, gv[i]);
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            ag[i][j] = 0.f; ab[i][j] = 0.f;
            if (COLS) { ad[i][j] = 0.f; ae[i][j] = 0.f; }
        }
    }
    // All three inputs of a row are requested together, and a row ahead: while a row is reduced and stored the next one
    // is in flight (held as loaded, widened to fp32 when its turn comes).
    Raw8<T> pd[NORM_BWD_MAXC], px[NORM_BWD_MAXC], pr[NORM_BWD_MAXC];
    auto request = [&](size_t row) {
#pragma unroll
        for (int i = 0; i < NORM_BWD_MAXC; ++i) {
            const int c = (threadIdx.x + i * 256) * 8;
            if (c < H && row < (size_t)nrows) {
                load_raw8(d_out + row * H + c, pd[i]);
                load_raw8(x + row * H + c, px[i]);
                load_raw8(d_res + row * H + c, pr[i]);
            }
        }
    };
    request(blockIdx.x);
    for (size_t row = blockIdx.x; row < (size_t)nrows; row += gridDim.x) {
        const float r = rstd[row];
        const float mu = LN ? mean[row] : 0.f;
        float dv[NORM_BWD_MAXC][8], xh[NORM_BWD_MAXC][8], rv[NORM_BWD_MAXC][8];
        float s0 = 0.f, s1 = 0.f;
#pragma unroll
        for (int i = 0; i < NORM_BWD_MAXC; ++i) {
            if ((threadIdx.x + i * 256) * 8 < H) { unpack8(pd[i], dv[i]); unpack8(px[i], xh[i]); unpack8(pr[i], rv[i]); }
        }
        request(row + gridDim.x);
#pragma unroll
        for (int i = 0; i < NORM_BWD_MAXC; ++i) {
            const int c = (threadIdx.x + i * 256) * 8;
            if (c < H) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    xh[i][j] = (xh[i][j] - mu) * r;
                    ag[i][j] += dv[i][j] * xh[i][j];
                    ab[i][j] += dv[i][j];
                    dv[i][j] *= gv[i][j];          // ghat
                    s0 += dv[i][j];
                    s1 += dv[i][j] * xh[i][j];
                }
            }
        }
        s1 = block_sum<4>(s1, red) / H;
        s0 = LN ? block_sum<4>(s0, red) / H : 0.f;
#pragma unroll
        for (int i = 0; i < NORM_BWD_MAXC; ++i) {
            const int c = (threadIdx.x + i * 256) * 8;
            if (c < H) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    if (COLS) ae[i][j] += rv[i][j];
                    rv[i][j] += r * (dv[i][j] - s0 - xh[i][j] * s1);
                    if (COLS) ad[i][j] += rv[i][j];
                }
                store8(d_in + row * H + c, rv[i]);      // a plain store: the streaming form is slower here (46 -> 49.5 us)
            }
        }
    }
#pragma unroll
    for (int i = 0; i < NORM_BWD_MAXC; ++i) {
        const int c = (threadIdx.x + i * 256) * 8;
        if (c < H) {
            if (part_g) store8(part_g + (size_t)blockIdx.x * H + c, ag[i]);
            if (LN && part_b) store8(part_b + (size_t)blockIdx.x * H + c, ab[i]);
            if (COLS && part_din) store8(part_din + (size_t)blockIdx.x * H + c, ad[i]);
            if (COLS && part_dres) store8(part_dres + (size_t)blockIdx.x * H + c, ae[i]);
        }
    }
}

hipError_t norm_bwd(int dtype, bool layernorm, const void *d_out, const void *x, const void *g,
                    const float *mean, const float *rstd, const void *d_res, void *d_in, float *part_g,
                    float *part_b, float *part_din, float *part_dres, int T, int H, hipStream_t st) {
    if (T == 0) return hipSuccess;
    if (H > 256 * 8 * NORM_BWD_MAXC) return hipErrorInvalidValue;
    const int grid = norm_bwd_blocks(T, H);
    const bool cols = part_din || part_dres;
#define L2(TT, LNV, MC, CV) norm_bwd_kernel<TT, LNV, MC, CV><<<grid, 256, 0, st>>>((const TT *)d_out, (const TT *)x, (const TT *)g, mean, rstd, (const TT *)d_res, (TT *)d_in, part_g, part_b, part_din, part_dres, T, H)
#define L1(TT, LNV, MC) do { if (cols) L2(TT, LNV, MC, true); else L2(TT, LNV, MC, false); } while (0)
#define L(TT, LNV) do { if (H <= 2048) L1(TT, LNV, 1); else if (H <= 4096) L1(TT, LNV, 2); else L1(TT, LNV, 4); } while (0)
    if (dtype == DT_F32) { if (layernorm) L(float, true); else L(float, false); }
    else { if (layernorm) L(bf16_t, true); else L(bf16_t, false); }
#undef L2
#undef L1
#undef L
    return hipGetLastError();
}

// ---- partial-sum reduction -----------------------------------------------------------
// 32 columns per workgroup.  Vector form (N a multiple of 4): 8 lanes cover the 32 columns with 16 bytes each and
// 32 row lanes walk the partial rows; scalar form: 32 column lanes, 8 row lanes.  Both combine through LDS in a
// fixed order.
template <typename T>
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float *__restrict__ part, int rows, int N,
                                                              T *__restrict__ out, bool accumulate) {
    __shared__ float red[8][33];
    const int c = blockIdx.x * 32 + (threadIdx.x & 31), rl = threadIdx.x >> 5;
    float s = 0.f;
    if (c < N)
        for (int r = rl; r < rows; r += 8) s += part[(size_t)r * N + c];
    red[rl][threadIdx.x & 31] = s;
    __syncthreads();
    if (rl == 0 && c < N) {
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) t += red[i][threadIdx.x];
        if (accumulate) t += Elem<T>::load(out + c);
        Elem<T>::store(out + c, t);
    }
}

template <typename T>
__global__ __launch_bounds__(256) void reduce_partials_vec_kernel(const float *__restrict__ part, int rows, int N,
                                                                  T *__restrict__ out, bool accumulate) {
    __shared__ float red[32][36];
    const int cl = threadIdx.x & 7, rl = threadIdx.x >> 3;
    const int c = blockIdx.x * 32 + cl * 4;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (c < N) {
        // eight rows in flight per thread: a thread's rows are 32 apart, and one load at a time leaves the kernel waiting
        // on memory latency (8 arrays of a few megabytes took 20 us)
        f32x4 t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = s;
        int r = rl;
        for (; r + 7 * 32 < rows; r += 256) {
            const float *q = part + (size_t)r * N + c;
            f32x4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const f32x4 *>(q + (size_t)(32 * u) * N);
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] += v[u];
        }
        for (; r < rows; r += 32) t[0] += *reinterpret_cast<const f32x4 *>(part + (size_t)r * N + c);
        s = ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
    }
    *reinterpret_cast<f32x4 *>(&red[rl][cl * 4]) = s;
    __syncthreads();
    const int oc = blockIdx.x * 32 + threadIdx.x;
    if (threadIdx.x < 32 && oc < N) {
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < 32; ++i) t += red[i][threadIdx.x];
        if (accumulate) t += Elem<T>::load(out + oc);
        Elem<T>::store(out + oc, t);
    }
}

hipError_t reduce_partials(int dtype, const float *part, int rows, int N, void *out, bool accumulate,
                           hipStream_t st) {
    if (N == 0) return hipSuccess;
    const int grid = ceil_div(N, 32);
    if (N % 4 == 0) {
        if (dtype == DT_F32) reduce_partials_vec_kernel<float><<<grid, 256, 0, st>>>(part, rows, N, (float *)out, accumulate);
        else reduce_partials_vec_kernel<bf16_t><<<grid, 256, 0, st>>>(part, rows, N, (bf16_t *)out, accumulate);
    } else {
        if (dtype == DT_F32) reduce_partials_kernel<float><<<grid, 256, 0, st>>>(part, rows, N, (float *)out, accumulate);
        else reduce_partials_kernel<bf16_t><<<grid, 256, 0, st>>>(part, rows, N, (bf16_t *)out, accumulate);
    }
    return hipGetLastError();
}

// Up to eight reductions of different shapes in one launch (blockIdx.y picks the job): everything a backward pass leaves
// behind as partial sums -- gain and bias gradients of both normalisations, the bias gradients of the four linears --
// is added up by one kernel at the end of the pass instead of by one launch where each array is produced.
struct ReduceJobSet { const float *part[8]; void *out[8]; int rows[8]; int N[8]; };
template <typename T>
__global__ __launch_bounds__(256) void reduce_jobs_kernel(ReduceJobSet set, bool accumulate) {
    __shared__ float red[32][36];
    const int N = set.N[blockIdx.y], rows = set.rows[blockIdx.y];
    if (blockIdx.x * 32 >= N) return;                                 // the grid is as wide as the widest job
    const float *part = set.part[blockIdx.y];
    T *out = (T *)set.out[blockIdx.y];
    const int cl = threadIdx.x & 7, rl = threadIdx.x >> 3;
    const int c = blockIdx.x * 32 + cl * 4;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    if (c < N) {
        // eight rows in flight per thread: a thread's rows are 32 apart, and one load at a time leaves the kernel waiting
        // on memory latency (8 arrays of a few megabytes took 20 us)
        f32x4 t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = s;
        int r = rl;
        for (; r + 7 * 32 < rows; r += 256) {
            const float *q = part + (size_t)r * N + c;
            f32x4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = *reinterpret_cast<const f32x4 *>(q + (size_t)(32 * u) * N);
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] += v[u];
        }
        for (; r < rows; r += 32) t[0] += *reinterpret_cast<const f32x4 *>(part + (size_t)r * N + c);
        s = ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
    }
    *reinterpret_cast<f32x4 *>(&red[rl][cl * 4]) = s;
    __syncthreads();
    const int oc = blockIdx.x * 32 + threadIdx.x;
    if (threadIdx.x < 32 && oc < N) {
        float t = 0.f;
#pragma unroll
        for (int i = 0; i < 32; ++i) t += red[i][threadIdx.x];
        if (accumulate) t += Elem<T>::load(out + oc);
        Elem<T>::store(out + oc, t);
    }
}

hipError_t reduce_jobs(int dtype, const ReduceJob *jobs, int n, bool accumulate, hipStream_t st) {
    ReduceJobSet set = {};
    int m = 0, widest = 0;
    bool quads = true;
    for (int i = 0; i < n && m < 8; ++i) {
        if (!jobs[i].part || !jobs[i].out || jobs[i].N <= 0) continue;
        set.part[m] = jobs[i].part; set.out[m] = jobs[i].out; set.rows[m] = jobs[i].rows; set.N[m] = jobs[i].N;
        widest = jobs[i].N > widest ? jobs[i].N : widest;
        quads = quads && jobs[i].N % 4 == 0;
        ++m;
    }
    if (m == 0) return hipSuccess;
    if (!quads) {                                  // the vector form needs whole quads: one launch each
        for (int i = 0; i < m; ++i) {
            hipError_t e = reduce_partials(dtype, set.part[i], set.rows[i], set.N[i], set.out[i], accumulate, st);
            if (e != hipSuccess) return e;
        }
        return hipSuccess;
    }
    dim3 grid(ceil_div(widest, 32), m);
    if (dtype == DT_F32) reduce_jobs_kernel<float><<<grid, 256, 0, st>>>(set, accumulate);
    else reduce_jobs_kernel<bf16_t><<<grid, 256, 0, st>>>(set, accumulate);
    return hipGetLastError();
}

// ---- column sums (bias gradients) ----------------------------------------------------
constexpr int COLSUM_ROWS = 16;            // rows per workgroup: short slabs, so that a [T, N] pass has T N / 32768 workgroups
int colsum_slabs(int T) { return T > 0 ? ceil_div(T, COLSUM_ROWS) : 1; }

template <typename T>
__global__ __launch_bounds__(256) void colsum_kernel(const T *__restrict__ in, int nrows, int N, int ld,
                                                     float *__restrict__ part) {
    const int c = (blockIdx.x * 256 + threadIdx.x) * 8;
    if (c >= N) return;
    const int r0 = blockIdx.y * COLSUM_ROWS;
    const int r1 = min(nrows, r0 + COLSUM_ROWS);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int r = r0; r < r1; r += 8) {              // 8 rows requested before the first is added
        float v[8][8];
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (r + k < r1) load8(in + (size_t)(r + k) * ld + c, v[k]);
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (r + k < r1) {
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] += v[k][j];
            }
    }
    store8(part + (size_t)blockIdx.y * N + c, acc);
}

hipError_t colsum_partials(int dtype, const void *in, int T, int N, int ld, float *part, hipStream_t st) {
    if (T == 0 || N == 0) return hipSuccess;
    dim3 grid(ceil_div(N, 2048), colsum_slabs(T));
    if (dtype == DT_F32) colsum_kernel<float><<<grid, 256, 0, st>>>((const float *)in, T, N, ld, part);
    else colsum_kernel<bf16_t><<<grid, 256, 0, st>>>((const bf16_t *)in, T, N, ld, part);
    return hipGetLastError();
}

// ---- rotary embedding, in place ------------------------------------------------------
// Heads [0, n_rot_heads) of every row (the q heads then the k heads) are rotated on the pair
// (i, i + d/2) by the tabulated angle of the token's position in its segment.  inverse = the
// transposed rotation (backward pass).
template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(T *__restrict__ qkv, int ld, int ntok, int n_rot_heads, int d,
                                                   const float2 *__restrict__ cs, float sgn) {
    const int half = d >> 1, cpp = half >> 3;                    // 8-wide chunks per half head
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    const long total = (long)ntok * n_rot_heads * cpp;
    if (idx >= total) return;
    const int ch = (int)(idx % cpp);
    const int h = (int)((idx / cpp) % n_rot_heads);
    const long t = idx / ((long)cpp * n_rot_heads);
    T *p = qkv + t * ld + h * d + ch * 8;
    float lo[8], hi[8];
    load8(p, lo);
    load8(p + half, hi);
    const float2 *c = cs + t * half + ch * 8;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float co = c[j].x, si = sgn * c[j].y;
        const float a = lo[j] * co - hi[j] * si, b = hi[j] * co + lo[j] * si;
        lo[j] = a; hi[j] = b;
    }
    store8(p, lo);
    store8(p + half, hi);
}

hipError_t rope_inplace(int dtype, void *qkv, int ld, int T, int n_rot_heads, int d, const float2 *rope_cs,
                        bool inverse, hipStream_t st) {
    const long total = (long)T * n_rot_heads * (d / 16);
    if (total == 0) return hipSuccess;
    const float sgn = inverse ? -1.f : 1.f;
    if (dtype == DT_F32) rope_kernel<float><<<ceil_div(total, 256), 256, 0, st>>>((float *)qkv, ld, T, n_rot_heads, d, rope_cs, sgn);
    else rope_kernel<bf16_t><<<ceil_div(total, 256), 256, 0, st>>>((bf16_t *)qkv, ld, T, n_rot_heads, d, rope_cs, sgn);
    return hipGetLastError();
}

// ---- SwiGLU --------------------------------------------------------------------------
// gu[T, 2F] = [gate | up];  m = gate * sigmoid(gate) * up.
// 1 / (1 + exp(-x)) with the hardware exponential and reciprocal (each within an fp32 rounding or two; the library's
// expf and the IEEE division take some twenty instructions more per element)
__device__ __forceinline__ float sigmoid_fast(float x) {
    return __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(x * -1.4426950408889634f));
}
template <typename T>
__global__ __launch_bounds__(256) void swiglu_fwd_kernel(const T *__restrict__ gu, T *__restrict__ m, long nchunks, int F) {
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= nchunks) return;
    const int cpr = F >> 3;
    const long t = idx / cpr;
    const int c = (int)(idx % cpr) * 8;
    float g[8], u[8];
    load8_stream(gu + t * 2 * F + c, g);
    load8_stream(gu + t * 2 * F + F + c, u);
#pragma unroll
    for (int j = 0; j < 8; ++j) g[j] = g[j] * sigmoid_fast(g[j]) * u[j];
    store8_stream(m + t * F + c, g);
}

// d_gate = d_m * up * s * (1 + gate * (1 - s)),  d_up = d_m * gate * s,  s = sigmoid(gate).
template <typename T>
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const T *__restrict__ d_m, const T *__restrict__ gu,
                                                         T *__restrict__ d_gu, long nchunks, int F) {
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= nchunks) return;
    const int cpr = F >> 3;
    const long t = idx / cpr;
    const int c = (int)(idx % cpr) * 8;
    float g[8], u[8], dm[8];
    load8_stream(gu + t * 2 * F + c, g);
    load8_stream(gu + t * 2 * F + F + c, u);
    load8_stream(d_m + t * F + c, dm);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const float s = 1.f / (1.f + expf(-g[j]));      // the library forms on purpose: with sigmoid_fast this kernel runs 6 % slower (141 -> 150 us)
        const float dg = dm[j] * u[j] * s * (1.f + g[j] * (1.f - s));
        u[j] = dm[j] * g[j] * s;
        g[j] = dg;
    }
    store8_stream(d_gu + t * 2 * F + c, g);
    store8_stream(d_gu + t * 2 * F + F + c, u);
}

hipError_t swiglu_fwd(int dtype, const void *gu, void *m, int T, int F, hipStream_t st) {
    const long n = (long)T * (F / 8);
    if (n == 0) return hipSuccess;
    if (dtype == DT_F32) swiglu_fwd_kernel<float><<<ceil_div(n, 256), 256, 0, st>>>((const float *)gu, (float *)m, n, F);
    else swiglu_fwd_kernel<bf16_t><<<ceil_div(n, 256), 256, 0, st>>>((const bf16_t *)gu, (bf16_t *)m, n, F);
    return hipGetLastError();
}
hipError_t swiglu_bwd(int dtype, const void *d_m, const void *gu, void *d_gu, int T, int F, hipStream_t st) {
    const long n = (long)T * (F / 8);
    if (n == 0) return hipSuccess;
    if (dtype == DT_F32) swiglu_bwd_kernel<float><<<ceil_div(n, 256), 256, 0, st>>>((const float *)d_m, (const float *)gu, (float *)d_gu, n, F);
    else swiglu_bwd_kernel<bf16_t><<<ceil_div(n, 256), 256, 0, st>>>((const bf16_t *)d_m, (const bf16_t *)gu, (bf16_t *)d_gu, n, F);
    return hipGetLastError();
}

// ---- GELU (erf form) -----------------------------------------------------------------
// Phi(v) and phi(v) of the standard normal distribution.  The library erff costs some forty vector instructions, which
// made these kernels bound by the vector ALUs (GELU backward ran at 3.6 TB/s); this is the five-term rational
// approximation of Abramowitz & Stegun 7.1.26, erf(x) = 1 - (a1 t + ... + a5 t^5) exp(-x^2), t = 1 / (1 + p x), x >= 0,
// absolute error 1.5e-7, whose exponential exp(-v^2 / 2) is phi's as well: a dozen instructions for both.  In fp32
// arithmetic Phi comes out within 3e-7 (absolute; an fp32 rounding of a value near 1 is 6e-8).
__device__ __forceinline__ void normal_cdf_pdf(float v, float &cdf, float &pdf) {
    const float e = __builtin_amdgcn_exp2f(v * v * -0.72134752044448170f);            // exp(-v^2 / 2)
    const float t = __builtin_amdgcn_rcpf(fmaf(0.23164189f, fabsf(v), 1.f));              // p / sqrt(2) = 0.3275911 / 1.41421356
    const float poly = ((((1.061405429f * t - 1.453152027f) * t + 1.421413741f) * t - 0.284496736f) * t + 0.254829592f) * t;
    const float h = 0.5f * poly * e;                                                     // the smaller tail
    cdf = v >= 0.f ? 1.f - h : h;
    pdf = 0.3989422804014327f * e;
}
template <typename T>
__global__ __launch_bounds__(256) void gelu_fwd_kernel(const T *__restrict__ z, T *__restrict__ a, long nchunks) {
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= nchunks) return;
    float v[8];
    load8(z + idx * 8, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        float cdf, pdf;
        normal_cdf_pdf(v[j], cdf, pdf);
        v[j] *= cdf;
    }
    store8(a + idx * 8, v);
}
// gelu'(z) = Phi(z) + z * phi(z)
template <typename T>
__global__ __launch_bounds__(256) void gelu_bwd_kernel(const T *__restrict__ d_a, const T *__restrict__ z,
                                                       T *__restrict__ d_z, long nchunks) {
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    if (idx >= nchunks) return;
    float v[8], g[8];
    load8(z + idx * 8, v);
    load8(d_a + idx * 8, g);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        float cdf, pdf;
        normal_cdf_pdf(v[j], cdf, pdf);
        v[j] = g[j] * (cdf + v[j] * pdf);
    }
    store8(d_z + idx * 8, v);
}

// The same over [nrows, N] with the column sums of d_z (the bias gradient of the linear in front of the activation):
// a thread owns 8 columns of a slab of COLSUM_ROWS rows; part[slab, N] receives the slab's sums.
template <typename T>
__global__ __launch_bounds__(256) void gelu_bwd_colsum_kernel(const T *__restrict__ d_a, const T *__restrict__ z,
                                                              T *__restrict__ d_z, int nrows, int N,
                                                              float *__restrict__ part) {
    const int c = (blockIdx.x * 256 + threadIdx.x) * 8;
    if (c >= N) return;
    const int r0 = blockIdx.y * COLSUM_ROWS, r1 = min(nrows, r0 + COLSUM_ROWS);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int r = r0; r < r1; r += 4) {
        float v[4][8], g[4][8];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (r + k < r1) { load8(z + (size_t)(r + k) * N + c, v[k]); load8(d_a + (size_t)(r + k) * N + c, g[k]); }
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (r + k < r1) {
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    float cdf, pdf;
                    normal_cdf_pdf(v[k][j], cdf, pdf);
                    v[k][j] = g[k][j] * (cdf + v[k][j] * pdf);
                }
                store8(d_z + (size_t)(r + k) * N + c, v[k]);
#pragma unroll
                for (int j = 0; j < 8; ++j) acc[j] += v[k][j];
            }
    }
    store8(part + (size_t)blockIdx.y * N + c, acc);
}

hipError_t gelu_fwd(int dtype, const void *z, void *a, long n, hipStream_t st) {
    const long nc = n / 8;
    if (nc == 0) return hipSuccess;
    if (dtype == DT_F32) gelu_fwd_kernel<float><<<ceil_div(nc, 256), 256, 0, st>>>((const float *)z, (float *)a, nc);
    else gelu_fwd_kernel<bf16_t><<<ceil_div(nc, 256), 256, 0, st>>>((const bf16_t *)z, (bf16_t *)a, nc);
    return hipGetLastError();
}
hipError_t gelu_bwd_colsum(int dtype, const void *d_a, const void *z, void *d_z, int T, int N, float *part, hipStream_t st) {
    if (T == 0 || N == 0) return hipSuccess;
    dim3 grid(ceil_div(N, 2048), colsum_slabs(T));
    if (dtype == DT_F32) gelu_bwd_colsum_kernel<float><<<grid, 256, 0, st>>>((const float *)d_a, (const float *)z, (float *)d_z, T, N, part);
    else gelu_bwd_colsum_kernel<bf16_t><<<grid, 256, 0, st>>>((const bf16_t *)d_a, (const bf16_t *)z, (bf16_t *)d_z, T, N, part);
    return hipGetLastError();
}
hipError_t gelu_bwd(int dtype, const void *d_a, const void *z, void *d_z, long n, hipStream_t st) {
    const long nc = n / 8;
    if (nc == 0) return hipSuccess;
    if (dtype == DT_F32) gelu_bwd_kernel<float><<<ceil_div(nc, 256), 256, 0, st>>>((const float *)d_a, (const float *)z, (float *)d_z, nc);
    else gelu_bwd_kernel<bf16_t><<<ceil_div(nc, 256), 256, 0, st>>>((const bf16_t *)d_a, (const bf16_t *)z, (bf16_t *)d_z, nc);
    return hipGetLastError();
}

}  // namespace mmt
