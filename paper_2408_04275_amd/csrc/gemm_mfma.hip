// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
//   C[M,N] (+)= opA(A) . opB(B) (+ bias[N]) (+ residual[M,N])
//
// Tiling.  One 256-thread workgroup (4 wavefronts, one per SIMD) owns a 256x256 tile of C;
// each wavefront owns a 128x128 quadrant as 4x4 MFMA tiles of 32x32 (256 accumulator
// registers per lane).  K advances in slices of 64 through a double-buffered LDS stage of
// 2 x (256x64 A + 256x64 B) bf16 = 128 KiB of the CU's 160 KiB.
//
// LDS layout.  Both operand tiles are kept "K-contiguous": row = m (or n), 64 k-values =
// 128 bytes = eight 16-byte units per row.  Unit u of row r is stored at unit position
// u ^ ((r ^ (r >> 3)) & 7), which spreads over all banks (a) the MFMA fragment reads (32 lanes
// = 32 consecutive rows, same unit), (b) the row-major tile writes (8 lanes = the 8 units of
// one row) and (c) the transposed tile writes (lanes 8 rows apart, same unit).
//
// Global -> LDS.  Operands whose contraction index is contiguous in memory (A of NT/NN, B of
// NT) are copied 16 bytes per lane.  Operands whose contraction index is the row index (B of
// NN, A and B of TN) are read 16 bytes per lane along their contiguous direction as 8x8
// blocks and transposed in registers (byte permutes) before the LDS write, so weight- and
// input-gradient GEMMs need no transposed copies in HBM.  Out-of-range rows and k are zero-filled.
//
// Epilogue.  Accumulators go through a per-wavefront fp32 LDS staging area so that C,
// residual and bias are accessed as full 16-byte row-major vectors; bias / residual / previous
// C (accumulate) are added in fp32 before the single rounding to bf16.
//
// Workgroup -> tile map.  Workgroups are dispatched round-robin over the 8 XCDs, each with
// its own L2; ids are remapped so that each XCD works on a contiguous run of tiles, ordered in
// column-major groups of 8 tile-rows so that concurrently resident tiles share A and B panels.
#include "kernels.h"

namespace mmt {

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int TILE_BYTES = BM * BK * 2;          // 32 KiB per operand tile
constexpr int STAGE_BYTES = 2 * TILE_BYTES;
constexpr int SMEM_BYTES = 2 * STAGE_BYTES;      // 128 KiB
constexpr int EPI_PITCH = 128 + 4;               // floats per staged row
constexpr int GROUP_M = 8;

struct GemmP {
    int M, N, K;
    const bf16_t *A; int lda;
    const bf16_t *B; int ldb;
    bf16_t *C; int ldc;
    const bf16_t *bias;
    const bf16_t *residual;
    int accumulate;
    int tiles_m, tiles_n;
};

__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }

// K-contiguous operand: X[rows, K] row-major.  Thread t copies unit (t & 7) of rows (t >> 3) + 32 i.
struct LoaderKC {
    uint4 r[8];
    __device__ __forceinline__ void load(const bf16_t *X, int ld, int row0, int nrows, int k0, int K) {
        const int c = threadIdx.x & 7, rr = threadIdx.x >> 3;
        const bool kok = k0 + c * 8 < K;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = row0 + rr + 32 * i;
            r[i] = make_uint4(0, 0, 0, 0);
            if (kok && row < nrows) r[i] = *reinterpret_cast<const uint4 *>(X + (size_t)row * ld + k0 + c * 8);
        }
    }
    __device__ __forceinline__ void store(uint8_t *tile) const {
        const int c = threadIdx.x & 7, rr = threadIdx.x >> 3;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int row = rr + 32 * i;
            *reinterpret_cast<uint4 *>(tile + (row * 8 + (c ^ swz(row))) * 16) = r[i];
        }
    }
};

// K-strided operand: X[K, rows] row-major.  Thread t owns the 8(k) x 8(row) block with
// row block (t & 31) and k block (t >> 5); it is transposed in registers on the way to LDS.
struct LoaderKS {
    uint4 r[8];
    __device__ __forceinline__ void load(const bf16_t *X, int ld, int row0, int nrows, int k0, int K) {
        const int rb = threadIdx.x & 31, kb = threadIdx.x >> 5;
        const bool rok = row0 + rb * 8 < nrows;
#pragma unroll
        for (int kk = 0; kk < 8; ++kk) {
            const int k = k0 + kb * 8 + kk;
            r[kk] = make_uint4(0, 0, 0, 0);
            if (rok && k < K) r[kk] = *reinterpret_cast<const uint4 *>(X + (size_t)k * ld + row0 + rb * 8);
        }
    }
    __device__ __forceinline__ void store(uint8_t *tile) const {
        const int rb = threadIdx.x & 31, kb = threadIdx.x >> 5;
        const uint32_t *w = reinterpret_cast<const uint32_t *>(r);   // w[kk * 4 + j]: rows 2j, 2j+1 at k = kk
#pragma unroll
        for (int rr = 0; rr < 8; ++rr) {
            const uint32_t sel = (rr & 1) ? 0x07060302u : 0x05040100u;
            uint4 o;
            o.x = __builtin_amdgcn_perm(w[1 * 4 + (rr >> 1)], w[0 * 4 + (rr >> 1)], sel);
            o.y = __builtin_amdgcn_perm(w[3 * 4 + (rr >> 1)], w[2 * 4 + (rr >> 1)], sel);
            o.z = __builtin_amdgcn_perm(w[5 * 4 + (rr >> 1)], w[4 * 4 + (rr >> 1)], sel);
            o.w = __builtin_amdgcn_perm(w[7 * 4 + (rr >> 1)], w[6 * 4 + (rr >> 1)], sel);
            const int row = rb * 8 + rr;
            *reinterpret_cast<uint4 *>(tile + (row * 8 + (kb ^ swz(row))) * 16) = o;
        }
    }
};

template <bool KC> struct LoaderSel { typedef LoaderKC type; };
template <> struct LoaderSel<false> { typedef LoaderKS type; };

template <bool A_KC, bool B_KC>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_mfma_kernel(const GemmP p) {
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];

    // ---- workgroup -> tile
    int tm, tn;
    {
        const int nb = gridDim.x, b = blockIdx.x;
        const int xcd = b & 7, q = b >> 3, per = nb >> 3, rem = nb & 7;
        const int logical = xcd < rem ? xcd * (per + 1) + q : rem * (per + 1) + (xcd - rem) * per + q;
        const int width = GROUP_M * p.tiles_n;
        const int group = logical / width, first_m = group * GROUP_M;
        const int gsize = min(p.tiles_m - first_m, GROUP_M);
        tm = first_m + (logical % width) % gsize;
        tn = (logical % width) / gsize;
    }
    const int m0 = tm * BM, n0 = tn * BN;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    typename LoaderSel<A_KC>::type la;
    typename LoaderSel<B_KC>::type lb;

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    // fragment addressing: lane reads row (lane & 31) of a 32-row block, unit ks*2 + (lane >> 5)
    const int frow = lane & 31, fhalf = lane >> 5;
    int a_off[4], b_off[4], a_sw[4], b_sw[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int ra = wm * 128 + i * 32 + frow, rb = wn * 128 + i * 32 + frow;
        a_off[i] = ra * 128; a_sw[i] = swz(ra);
        b_off[i] = rb * 128; b_sw[i] = swz(rb);
    }

    const int nk = (p.K + BK - 1) / BK;
    la.load(p.A, p.lda, m0, p.M, 0, p.K);
    lb.load(p.B, p.ldb, n0, p.N, 0, p.K);
    la.store(smem);
    lb.store(smem + TILE_BYTES);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
        const uint8_t *sa = smem + (kt & 1) * STAGE_BYTES;
        const uint8_t *sb = sa + TILE_BYTES;
        const bool more = kt + 1 < nk;
        if (more) {
            la.load(p.A, p.lda, m0, p.M, (kt + 1) * BK, p.K);
            lb.load(p.B, p.ldb, n0, p.N, (kt + 1) * BK, p.K);
        }
        bf16x8 fa[2][4], fb[2][4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            fa[0][i] = *reinterpret_cast<const bf16x8 *>(sa + a_off[i] + ((fhalf ^ a_sw[i]) << 4));
            fb[0][i] = *reinterpret_cast<const bf16x8 *>(sb + b_off[i] + ((fhalf ^ b_sw[i]) << 4));
        }
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            if (ks < 3) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int u = (ks + 1) * 2 + fhalf;
                    fa[nxt][i] = *reinterpret_cast<const bf16x8 *>(sa + a_off[i] + ((u ^ a_sw[i]) << 4));
                    fb[nxt][i] = *reinterpret_cast<const bf16x8 *>(sb + b_off[i] + ((u ^ b_sw[i]) << 4));
                }
            }
            // operands swapped: the accumulator tile is held transposed (lane = m, registers run
            // over n), so that each lane owns 4 consecutive n per register quad for the epilogue.
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[cur][j], fa[cur][i], acc[i][j], 0, 0, 0);
        }
        if (more) {
            uint8_t *da = smem + ((kt + 1) & 1) * STAGE_BYTES;
            la.store(da);
            lb.store(da + TILE_BYTES);
        }
        __syncthreads();
    }

    // ---- epilogue: 32 rows x 128 columns at a time through this wavefront's staging area
    float *stg = reinterpret_cast<float *>(smem) + wave * (32 * EPI_PITCH);
    const int er = lane >> 4, ec = (lane & 15) * 8;      // read-back: row er + 4*pass, columns ec..ec+7
    const int gn = n0 + wn * 128 + ec;
    const bool nok = gn < p.N;
    float bv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (p.bias && nok) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(p.bias + gn);
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) { bv[2 * e] = __uint_as_float(w[e] << 16); bv[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u); }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                // accumulator register 4*gq + e  <->  n = 8*gq + 4*(lane >> 5) + e,  m = lane & 31
                float4 v = make_float4(acc[i][j][4 * gq], acc[i][j][4 * gq + 1], acc[i][j][4 * gq + 2], acc[i][j][4 * gq + 3]);
                *reinterpret_cast<float4 *>(stg + frow * EPI_PITCH + j * 32 + gq * 8 + fhalf * 4) = v;
            }
        __syncthreads();
#pragma unroll
        for (int pass = 0; pass < 8; ++pass) {
            const int r = pass * 4 + er;
            const int gm = m0 + wm * 128 + i * 32 + r;
            if (gm < p.M && nok) {
                const float4 v0 = *reinterpret_cast<const float4 *>(stg + r * EPI_PITCH + ec);
                const float4 v1 = *reinterpret_cast<const float4 *>(stg + r * EPI_PITCH + ec + 4);
                float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] += bv[e];
                const size_t off = (size_t)gm * p.ldc + gn;
                if (p.residual) {
                    const uint4 raw = *reinterpret_cast<const uint4 *>(p.residual + off);
                    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) { v[2 * e] += __uint_as_float(w[e] << 16); v[2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u); }
                }
                if (p.accumulate) {
                    const uint4 raw = *reinterpret_cast<const uint4 *>(p.C + off);
                    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) { v[2 * e] += __uint_as_float(w[e] << 16); v[2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u); }
                }
                uint4 o;
                o.x = pack_bf16x2(v[0], v[1]); o.y = pack_bf16x2(v[2], v[3]);
                o.z = pack_bf16x2(v[4], v[5]); o.w = pack_bf16x2(v[6], v[7]);
                *reinterpret_cast<uint4 *>(p.C + off) = o;
            }
        }
        __syncthreads();
    }
}

template <bool A_KC, bool B_KC>
hipError_t launch(const GemmP &p, hipStream_t st) {
    static bool configured = false;
    auto kern = gemm_mfma_kernel<A_KC, B_KC>;
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
        if (e != hipSuccess) return e;
        configured = true;
    }
    kern<<<p.tiles_m * p.tiles_n, 256, SMEM_BYTES, st>>>(p);
    return hipGetLastError();
}

}  // namespace

bool gemm_mfma_supported(const GemmArgs &g) {
    if (g.M <= 0 || g.N <= 0 || g.K <= 0) return false;
    if ((g.lda | g.ldb | g.ldc | g.N) & 7) return false;
    const bool a_kc = g.layout != GEMM_TN, b_kc = g.layout == GEMM_NT;
    if ((a_kc || b_kc) && (g.K & 7)) return false;
    if (!a_kc && (g.M & 7)) return false;
    const uintptr_t bits = (uintptr_t)g.A | (uintptr_t)g.B | (uintptr_t)g.C | (uintptr_t)g.bias | (uintptr_t)g.residual;
    return (bits & 15) == 0;
}

hipError_t gemm_mfma(const GemmArgs &g, hipStream_t st) {
    GemmP p;
    p.M = g.M; p.N = g.N; p.K = g.K;
    p.A = (const bf16_t *)g.A; p.lda = g.lda;
    p.B = (const bf16_t *)g.B; p.ldb = g.ldb;
    p.C = (bf16_t *)g.C; p.ldc = g.ldc;
    p.bias = (const bf16_t *)g.bias;
    p.residual = (const bf16_t *)g.residual;
    p.accumulate = g.accumulate ? 1 : 0;
    p.tiles_m = ceil_div(g.M, BM);
    p.tiles_n = ceil_div(g.N, BN);
    switch (g.layout) {
        case GEMM_NT: return launch<true, true>(p, st);
        case GEMM_NN: return launch<true, false>(p, st);
        default: return launch<false, false>(p, st);
    }
}

}  // namespace mmt
