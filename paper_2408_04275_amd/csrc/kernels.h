// Internal launch interface between the C-ABI layer (api.hip) and the kernel files.
// Every launcher enqueues on `st` and returns the launch status; none synchronises.
#pragma once
#include "common.h"

namespace mmt {

enum { DT_F32 = 0, DT_BF16 = 1 };
enum { GEMM_NT = 0, GEMM_NN = 1, GEMM_TN = 2 };
enum { MASK_CAUSAL = 0, MASK_BIDIR = 1 };

struct GemmArgs {
    int layout;                 // GEMM_NT / GEMM_NN / GEMM_TN
    int M, N, K;
    const void *A; int lda;
    const void *B; int ldb;
    void *C; int ldc;
    const void *bias;           // [N] or null
    const void *residual;       // [M, ldc] or null
    bool accumulate;            // C += result
    bool c_f32 = false;         // C is fp32 whatever the operands' dtype (bias / residual are not combined with it)
    // optional scratch for split-K (TN on the matrix cores only): fp32 partial products, 256-byte aligned
    void *split_ws = nullptr;
    size_t split_ws_bytes = 0;
    // measurement aid (matrix-core kernel only): when not null, device uint64[4]; the first workgroup stores the
    // shader-clock counter and the constant 100 MHz counter at its start ([0], [1]) and at its end ([2], [3])
    unsigned long long *clock_probe = nullptr;
};

// gemm_simple.hip: any dtype, any shape, LDS-tiled FMA kernel (the fp32 path).
hipError_t gemm_simple(int dtype, const GemmArgs &g, hipStream_t st);
// gemm_mfma.hip: bf16 MFMA kernel.  `supported` checks alignment requirements.
bool gemm_mfma_supported(const GemmArgs &g);
hipError_t gemm_mfma(const GemmArgs &g, hipStream_t st);
// Weight gradients with few output tiles (gemm_mfma_few_tiles: transposed-A layout, no bias / residual, at most 128 tiles of
// 256 x 256) computed together in one launch, none of them cut along K; up to 4, all with the same accumulate / c_f32.
bool gemm_mfma_few_tiles(const GemmArgs &g);
hipError_t gemm_mfma_group(const GemmArgs *gs, int n, hipStream_t st);

// Segment bookkeeping produced by prep_tokens():
//   tok_seg[t]  = index of the segment that holds token t
//   tok_info[t] = {start of that segment, end of that segment with bit 30 set if it is bidirectional}
struct AttnArgs {
    int T, S, nh, nkv, d;
    float scale;
    const int *cu;              // device [S+1]
    const uint8_t *modes;       // device [S] or null
    int default_mode;
    const int *tok_seg;         // device [T]
    const void *qkv; int ld_qkv;
    void *o;                    // [T, nh*d]
    float *lse;                 // [nh, T]
    const void *d_o;            // bwd: [T, nh*d]
    void *d_qkv;                // bwd: [T, ld_qkv]
    float *Dsum;                // bwd scratch: [nh, T]; D = rowsum(dO * O) per query and head (the matrix-core kernels keep -D there)
    // MFMA path: tok_info[t] = {segment start, segment end | (bidirectional ? 1 << 30 : 0)}
    const int2 *tok_info;
    // MFMA path, backward: when not null, the [T, d/2] (cos, sin) table of the rotary embedding; dQ and dK are
    // then rotated back in the kernels' epilogues (otherwise the caller does it afterwards)
    const float2 *rope_cs;
    // MFMA path: dispatch order of the query tiles (256 queries: forward, dQ) and of the key tiles (128
    // keys: dK/dV), heaviest first; use_order = 0 means index order (more tiles than the tables hold)
    int use_order;
    uint8_t order_q[64];
    uint8_t order_k[128];
    // MFMA path, measurement aid: when not null, device [3][1024] counters; every workgroup adds its run time
    // (100 MHz ticks) to the entry of the compute unit it ran on (forward: row 0, dQ: row 1, dK/dV: row 2)
    unsigned long long *cu_busy;
};
// reorder.hip (host): Algorithm 1 and the tile orders above
int intra_reorder(const double *sizes, int n, int m, int32_t *order, int32_t *group_begin, double *group_load);
void attn_tile_order(const int32_t *cu_host, const uint8_t *modes_host, int default_mode, int S, int T, AttnArgs &a);
// pipeline.hip (host): timeline of the one-forward-one-backward pipeline schedule and Algorithm 2.
// fwd / bwd: [p][l] durations by original microbatch index; order: [l] (null: identity); return 0 on success
int pipeline_1f1b(const double *fwd, const double *bwd, int p, int l, const int32_t *order, double *makespan,
                  double *intervals /* [l] or null */);
int inter_reorder(const double *fwd, const double *bwd, int p, int l, const double *sizes /* [l] or null */, int32_t *order,
                  double *intervals_seen /* [l] or null */, int32_t *n_seen /* or null */);
// attn_simple.hip: fp32 arithmetic on the vector ALUs, any storage dtype
hipError_t attn_simple_fwd(int dtype, const AttnArgs &a, hipStream_t st);
hipError_t attn_simple_bwd(int dtype, const AttnArgs &a, hipStream_t st);
// attn_mfma.hip: bf16 storage, matrix cores
hipError_t attn_mfma_fwd(const AttnArgs &a, hipStream_t st);
hipError_t attn_mfma_bwd(const AttnArgs &a, hipStream_t st);

// elementwise.hip
hipError_t prep_tokens(const int *cu, const uint8_t *modes, int default_mode, int S, int T, int *tok_seg,
                       int2 *tok_info, int d, float rope_base, float2 *rope_cs /* [T, d/2] or null */,
                       hipStream_t st);
hipError_t norm_fwd(int dtype, bool layernorm, const void *x, const void *g, const void *b, void *out,
                    float *mean, float *rstd, int T, int H, float eps, hipStream_t st);
// d_in = norm_bwd(d_out) + d_res;  gain/bias gradient partial sums go to part_g/part_b, the column sums of d_in
// and of d_res to part_din / part_dres ([norm_bwd_blocks(T, H), H] fp32 each; null = skip).
int norm_bwd_blocks(int T, int H);
hipError_t norm_bwd(int dtype, bool layernorm, const void *d_out, const void *x, const void *g,
                    const float *mean, const float *rstd, const void *d_res, void *d_in,
                    float *part_g, float *part_b, float *part_din, float *part_dres, int T, int H, hipStream_t st);
// out[c] (+)= sum_r part[r, c]
hipError_t reduce_partials(int dtype, const float *part, int rows, int N, void *out, bool accumulate,
                           hipStream_t st);
int colsum_slabs(int T);
// out[N] (+)= the sum of the rows of part[rows, N], for up to eight arrays of different shapes in one launch (null part or out: skipped)
struct ReduceJob { const float *part; void *out; int rows, N; };
hipError_t reduce_jobs(int dtype, const ReduceJob *jobs, int n, bool accumulate, hipStream_t st);
hipError_t colsum_partials(int dtype, const void *in, int T, int N, int ld, float *part, hipStream_t st);
hipError_t rope_inplace(int dtype, void *qkv, int ld, int T, int n_rot_heads, int d, const float2 *rope_cs,
                        bool inverse, hipStream_t st);
hipError_t swiglu_fwd(int dtype, const void *gu, void *m, int T, int F, hipStream_t st);
hipError_t swiglu_bwd(int dtype, const void *d_m, const void *gu, void *d_gu, int T, int F, hipStream_t st);
hipError_t gelu_fwd(int dtype, const void *z, void *a, long n, hipStream_t st);
hipError_t gelu_bwd(int dtype, const void *d_a, const void *z, void *d_z, long n, hipStream_t st);
// the same over [T, N] rows, with the column sums of d_z as partial sums part[colsum_slabs(T), N]
hipError_t gelu_bwd_colsum(int dtype, const void *d_a, const void *z, void *d_z, int T, int N, float *part, hipStream_t st);


// optimizer.hip: one AdamW step on fp32 master weights; omb = 1 - beta, inv_bias1 = 1 / (1 - beta1^t),
// inv_bias2 = 1 / (1 - beta2^t), all four evaluated in double by the caller
struct AdamArgs {
    float lr, beta1, beta2, omb1, omb2, eps, weight_decay, grad_scale, inv_bias1, inv_bias2;
    int zero_grad;
};
hipError_t adam_step(int param_dtype, size_t n, float *w, float *g, float *m, float *v, void *p, const AdamArgs &a,
                     hipStream_t st);

}  // namespace mmt
