// C-ABI of the library: argument validation (host only, before any HIP call), memory
// carving of ctx / workspace, and the launch sequence of one layer forward / backward.
#include "../../include/mmtrain.h"
#include "kernels.h"
#include <cmath>
#include <initializer_list>
#include <mutex>
#include <vector>

using namespace mmt;

namespace {

struct Bump {
    uint8_t *base;
    size_t off;
    template <typename T> T *take(size_t n) {
        off = (off + 255) & ~size_t(255);
        T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
        off += n * sizeof(T);
        return p;
    }
    void *take_elems(size_t n, int dtype) {
        return dtype == DT_F32 ? (void *)take<float>(n) : (void *)take<bf16_t>(n);
    }
};

struct Dims {
    int kind, dtype, H, nh, nkv, d, F, F1, nq, nk, nqkv;
    float eps, rope_base, scale;
};

// Saved activations.  Everything the backward pass reads is kept (the forward pass produces
// all of it anyway); nothing is recomputed.
struct Ctx {
    float *mean1, *rstd1, *mean2, *rstd2, *lse;
    int *tok_seg;
    int2 *tok_info;
    float2 *rope_cs;
    void *h1, *qkv, *o, *y1, *h2, *pre, *m;
};

struct BwdWs {
    void *d_m, *d_pre, *d_h, *d_y1, *d_o, *d_qkv;
    float *Dsum, *part_g, *part_b, *part_c, *part_din, *part_dres;      // partial sums of the second normalisation's backward pass and of fc1's bias
    float *part_g1, *part_b1, *part_c2;                                 // ... of the first normalisation's and of the QKV bias (all reduced at the end of the pass)
    void *split_ws; size_t split_bytes;     // fp32 partial products of split weight-gradient GEMMs
};

int check_desc(const mmtrain_layer_desc *desc, Dims &D) {
    if (!desc || desc->struct_size != sizeof(mmtrain_layer_desc)) return MMTRAIN_ERR_INVALID_ARG;
    if (desc->kind != MMTRAIN_DECODER && desc->kind != MMTRAIN_ENCODER) return MMTRAIN_ERR_INVALID_ARG;
    if (desc->dtype != MMTRAIN_F32 && desc->dtype != MMTRAIN_BF16) return MMTRAIN_ERR_INVALID_ARG;
    if (desc->hidden <= 0 || desc->n_heads <= 0 || desc->n_kv_heads <= 0 || desc->ffn_hidden <= 0)
        return MMTRAIN_ERR_INVALID_ARG;
    if (!(desc->norm_eps > 0.f) || desc->softmax_scale < 0.f) return MMTRAIN_ERR_INVALID_ARG;
    if (desc->kind == MMTRAIN_DECODER && !(desc->rope_base > 1.f)) return MMTRAIN_ERR_INVALID_ARG;
    // 64 and 128 are the kernels' native tile widths; other multiples of 16 up to 128 (80: ViT-Huge) run on
    // the matrix-core kernels with the head zero-padded in LDS and registers (bf16 storage only)
    if (desc->head_dim != 64 && desc->head_dim != 128 &&
        !(desc->dtype == MMTRAIN_BF16 && desc->head_dim >= 16 && desc->head_dim < 128 && desc->head_dim % 16 == 0))
        return MMTRAIN_ERR_UNSUPPORTED;
    if (desc->n_heads % desc->n_kv_heads) return MMTRAIN_ERR_UNSUPPORTED;
    if (desc->kind == MMTRAIN_ENCODER && desc->n_kv_heads != desc->n_heads) return MMTRAIN_ERR_UNSUPPORTED;
    if ((desc->hidden % 16) || (desc->ffn_hidden % 16)) return MMTRAIN_ERR_UNSUPPORTED;
    if (desc->hidden > 8192) return MMTRAIN_ERR_UNSUPPORTED;
    D.kind = desc->kind; D.dtype = desc->dtype; D.H = desc->hidden; D.nh = desc->n_heads;
    D.nkv = desc->n_kv_heads; D.d = desc->head_dim; D.F = desc->ffn_hidden;
    D.F1 = desc->kind == MMTRAIN_DECODER ? 2 * D.F : D.F;
    D.nq = D.nh * D.d; D.nk = D.nkv * D.d; D.nqkv = D.nq + 2 * D.nk;
    D.eps = desc->norm_eps; D.rope_base = desc->rope_base;
    D.scale = desc->softmax_scale > 0.f ? desc->softmax_scale : 1.0f / sqrtf((float)D.d);
    return MMTRAIN_OK;
}

int check_batch(const mmtrain_batch *b) {
    if (!b) return MMTRAIN_ERR_INVALID_ARG;
    if (b->total_tokens < 0 || b->n_segments < 0) return MMTRAIN_ERR_INVALID_ARG;
    if (b->mask_mode != MMTRAIN_MASK_CAUSAL && b->mask_mode != MMTRAIN_MASK_BIDIR) return MMTRAIN_ERR_INVALID_ARG;
    if (!b->cu_seqlens_host) return MMTRAIN_ERR_INVALID_ARG;
    if ((b->seg_mask_dev == nullptr) != (b->seg_mask_host == nullptr)) return MMTRAIN_ERR_INVALID_ARG;
    const int32_t *cu = b->cu_seqlens_host;
    if (cu[0] != 0) return MMTRAIN_ERR_BAD_SEGMENTS;
    for (int s = 0; s < b->n_segments; ++s)
        if (cu[s + 1] < cu[s]) return MMTRAIN_ERR_BAD_SEGMENTS;
    if (cu[b->n_segments] != b->total_tokens) return MMTRAIN_ERR_BAD_SEGMENTS;
    if (b->seg_mask_host)
        for (int s = 0; s < b->n_segments; ++s)
            if (b->seg_mask_host[s] > 1) return MMTRAIN_ERR_INVALID_ARG;
    if (b->total_tokens > 0 && !b->cu_seqlens_dev) return MMTRAIN_ERR_INVALID_ARG;
    return MMTRAIN_OK;
}

// The kernels move 16 bytes per lane (vector loads and stores, direct-to-LDS copies): every tensor pointer must be
// 16-byte aligned.  A misaligned one (a view such as tensor[1:]) is an argument error, not a memory fault.
bool misaligned(std::initializer_list<const void *> ptrs) {
    uintptr_t bits = 0;
    for (const void *p : ptrs) bits |= (uintptr_t)p;
    return (bits & 15) != 0;
}

int check_weights(const Dims &D, const mmtrain_layer_weights *w) {
    if (!w) return MMTRAIN_ERR_INVALID_ARG;
    if (!w->norm1_w || !w->w_qkv || !w->w_o || !w->norm2_w || !w->w_fc1 || !w->w_fc2) return MMTRAIN_ERR_INVALID_ARG;
    if (D.kind == MMTRAIN_ENCODER &&
        (!w->norm1_b || !w->b_qkv || !w->b_o || !w->norm2_b || !w->b_fc1 || !w->b_fc2))
        return MMTRAIN_ERR_INVALID_ARG;
    if (misaligned({w->norm1_w, w->norm1_b, w->w_qkv, w->b_qkv, w->w_o, w->b_o, w->norm2_w, w->norm2_b, w->w_fc1, w->b_fc1,
                    w->w_fc2, w->b_fc2}))
        return MMTRAIN_ERR_INVALID_ARG;
    return MMTRAIN_OK;
}

int check_grads(const mmtrain_layer_grads *g) {
    if (g && misaligned({g->norm1_w, g->norm1_b, g->w_qkv, g->b_qkv, g->w_o, g->b_o, g->norm2_w, g->norm2_b, g->w_fc1, g->b_fc1,
                         g->w_fc2, g->b_fc2}))
        return MMTRAIN_ERR_INVALID_ARG;
    return MMTRAIN_OK;
}

void carve_ctx(Bump &b, const Dims &D, size_t T, Ctx &c) {
    c.mean1 = b.take<float>(T); c.rstd1 = b.take<float>(T);
    c.mean2 = b.take<float>(T); c.rstd2 = b.take<float>(T);
    c.lse = b.take<float>(T * D.nh);
    c.tok_seg = b.take<int>(T);
    c.tok_info = b.take<int2>(T);
    c.rope_cs = D.kind == MMTRAIN_DECODER ? b.take<float2>(T * (D.d / 2)) : nullptr;
    c.h1 = b.take_elems(T * D.H, D.dtype);
    c.qkv = b.take_elems(T * D.nqkv, D.dtype);
    c.o = b.take_elems(T * D.nq, D.dtype);
    c.y1 = b.take_elems(T * D.H, D.dtype);
    c.h2 = b.take_elems(T * D.H, D.dtype);
    c.pre = b.take_elems(T * D.F1, D.dtype);
    c.m = b.take_elems(T * D.F, D.dtype);
}

// Scratch that lets an M x N gradient GEMM be cut along K in both ways the bf16 kernel knows: few output tiles
// (gemm_mfma_splits: up to 256 / tiles products of M x N, 32 at most), or a partly filled last round of tiles
// (gemm_mfma_tail_splits: never more than 256 blocks of 256 x 256).
size_t gemm_scratch_bytes(size_t M, size_t N) {
    const size_t tiles = ((M + 255) / 256) * ((N + 255) / 256);
    if (tiles > 128) return tiles % 256 && tiles % 256 <= 128 ? size_t(256) * 256 * 256 * 4 : 0;
    const size_t s = 256 / tiles < 32 ? 256 / tiles : 32;
    return s >= 2 ? s * M * N * 4 : 0;
}

void carve_bwd(Bump &b, const Dims &D, size_t T, BwdWs &w) {
    w.d_m = b.take_elems(T * D.F, D.dtype);
    w.d_pre = b.take_elems(T * D.F1, D.dtype);
    w.d_h = b.take_elems(T * D.H, D.dtype);
    w.d_y1 = b.take_elems(T * D.H, D.dtype);
    w.d_o = b.take_elems(T * D.nq, D.dtype);
    w.d_qkv = b.take_elems(T * D.nqkv, D.dtype);
    w.Dsum = b.take<float>(T * D.nh);
    w.part_g = b.take<float>((size_t)norm_bwd_blocks((int)T, D.H) * D.H);
    w.part_b = b.take<float>((size_t)norm_bwd_blocks((int)T, D.H) * D.H);
    const bool enc = D.kind == MMTRAIN_ENCODER;            // bias gradients that the normalisation's backward kernel sums
    w.part_din = enc ? b.take<float>((size_t)norm_bwd_blocks((int)T, D.H) * D.H) : nullptr;
    w.part_dres = enc ? b.take<float>((size_t)norm_bwd_blocks((int)T, D.H) * D.H) : nullptr;
    const int maxn = D.nqkv > D.F1 ? (D.nqkv > D.H ? D.nqkv : D.H) : (D.F1 > D.H ? D.F1 : D.H);
    w.part_c = b.take<float>((size_t)colsum_slabs((int)T) * maxn);
    w.part_g1 = b.take<float>((size_t)norm_bwd_blocks((int)T, D.H) * D.H);
    w.part_b1 = enc ? b.take<float>((size_t)norm_bwd_blocks((int)T, D.H) * D.H) : nullptr;
    w.part_c2 = enc ? b.take<float>((size_t)colsum_slabs((int)T) * D.nqkv) : nullptr;
    // scratch for the fp32 partial products of GEMMs that are cut along K (see gemm_scratch_bytes)
    auto need = [](size_t M, size_t N) -> size_t { return gemm_scratch_bytes(M, N); };
    size_t sb = 0;
    if (D.dtype == DT_BF16) {
        const size_t c[8] = {need(D.H, D.F), need(D.F1, D.H), need(D.H, D.nq), need(D.nqkv, D.H),
                             need(T, D.F), need(T, D.H), need(T, D.nq), 0};
        for (size_t v : c) sb = v > sb ? v : sb;
    }
    w.split_bytes = sb;
    w.split_ws = sb ? (void *)b.take<float>(sb / 4) : nullptr;
}

hipError_t gemm(int dtype, const GemmArgs &g, hipStream_t st);


// bf16 storage runs on the matrix cores; fp32 storage on the vector ALUs
hipError_t attn_fwd(int dtype, const AttnArgs &a, hipStream_t st) {
    return dtype == DT_BF16 ? attn_mfma_fwd(a, st) : attn_simple_fwd(dtype, a, st);
}
hipError_t attn_bwd(int dtype, const AttnArgs &a, hipStream_t st) {
    return dtype == DT_BF16 ? attn_mfma_bwd(a, st) : attn_simple_bwd(dtype, a, st);
}

GemmArgs f32out(GemmArgs g, bool on) { g.c_f32 = on; return g; }
GemmArgs splittable(GemmArgs g, void *ws, size_t bytes) { g.split_ws = ws; g.split_ws_bytes = bytes; return g; }

GemmArgs mk(int layout, int M, int N, int K, const void *A, int lda, const void *B, int ldb, void *C, int ldc,
            const void *bias = nullptr, const void *residual = nullptr, bool accumulate = false) {
    GemmArgs g;
    g.layout = layout; g.M = M; g.N = N; g.K = K; g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc;
    g.bias = bias; g.residual = residual; g.accumulate = accumulate;
    return g;
}

unsigned long long *g_attn_busy = nullptr;      // device [3][1024] or null: see mmtrain_profile_attn_busy

AttnArgs mk_attn(const Dims &D, const mmtrain_batch *b, const Ctx &c) {
    AttnArgs a = {};
    a.cu_busy = g_attn_busy;
    a.T = b->total_tokens; a.S = b->n_segments; a.nh = D.nh; a.nkv = D.nkv; a.d = D.d; a.scale = D.scale;
    a.cu = b->cu_seqlens_dev; a.modes = b->seg_mask_dev; a.default_mode = b->mask_mode;
    a.tok_seg = c.tok_seg; a.tok_info = c.tok_info; a.qkv = c.qkv; a.ld_qkv = D.nqkv; a.o = c.o; a.lse = c.lse;
    attn_tile_order(b->cu_seqlens_host, b->seg_mask_host, b->mask_mode, b->n_segments, b->total_tokens, a);
    return a;
}

__global__ void fill_zero_kernel(uint32_t *p, size_t nwords) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < nwords) p[i] = 0u;
}
hipError_t fill_zero(void *p, size_t elems, int dtype, hipStream_t st) {
    if (!p || elems == 0) return hipSuccess;
    const size_t bytes = elems * (dtype == DT_F32 ? 4 : 2);
    const size_t words = bytes / 4;            // all parameter tensors have an even element count
    fill_zero_kernel<<<ceil_div((long)words, 256), 256, 0, st>>>((uint32_t *)p, words);
    return hipGetLastError();
}

#define HIP_TRY(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) return MMTRAIN_ERR_HIP; } while (0)
// the same with the launch bracketed by the events of profiling class `kind` (when that class is enabled)
#define HIP_TRY_TIMED(kind, st, expr) do { ProfScope ps_((kind), (st)); hipError_t e_ = (expr); if (e_ != hipSuccess) return MMTRAIN_ERR_HIP; } while (0)

// ---- optional per-kernel-class timing with HIP events on the caller's stream -------------
struct Profiler {
    int mask = 0;                                  // bit k: class k is being timed
    struct Span { int kind; hipEvent_t a, b; };
    std::vector<Span> spans;
    std::vector<hipEvent_t> pool;
    hipEvent_t get() {
        if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
};
Profiler g_prof;

struct ProfScope {
    int kind; hipStream_t st; hipEvent_t a = nullptr, b = nullptr;
    ProfScope(int k, hipStream_t s) : kind(k), st(s) {
        if (!((g_prof.mask >> k) & 1)) return;
        a = g_prof.get(); b = g_prof.get();
        if (a && b) (void)hipEventRecord(a, st);
    }
    ~ProfScope() {
        if (!a || !b) return;
        (void)hipEventRecord(b, st);
        g_prof.spans.push_back({kind, a, b});
    }
};

unsigned long long *g_gemm_clock = nullptr;     // device uint64[4] or null: see mmtrain_profile_gemm_clock

hipError_t gemm(int dtype, const GemmArgs &g, hipStream_t st) {
    ProfScope ps(g.layout, st);                    // MMTRAIN_PROF_GEMM_NT / _NN / _TN
    if (dtype == DT_BF16 && gemm_mfma_supported(g)) {
        if (!g_gemm_clock) return gemm_mfma(g, st);
        GemmArgs probed = g;
        probed.clock_probe = g_gemm_clock;
        return gemm_mfma(probed, st);
    }
    return gemm_simple(dtype, g, st);
}

// Weight-gradient GEMMs of a backward pass whose outputs have few tiles are not launched where they stand but
// collected and run together at the end of the pass (gemm_mfma_group): their operands all live until then.
struct DeferredWgrads {
    GemmArgs g[4];
    int n = 0;
};
hipError_t wgrad(int dtype, const GemmArgs &g, DeferredWgrads &later, hipStream_t st) {
    if (dtype == DT_BF16 && later.n < 4 && gemm_mfma_few_tiles(g)) {
        later.g[later.n++] = g;
        return hipSuccess;
    }
    return gemm(dtype, g, st);
}
hipError_t run_deferred(const DeferredWgrads &later, hipStream_t st) {
    if (later.n == 0) return hipSuccess;
    ProfScope ps(MMTRAIN_PROF_GEMM_TN, st);
    return gemm_mfma_group(later.g, later.n, st);
}

}  // namespace

extern "C" {

const char *mmtrain_status_string(int status) {
    switch (status) {
        case MMTRAIN_OK: return "ok";
        case MMTRAIN_ERR_INVALID_ARG: return "invalid argument";
        case MMTRAIN_ERR_BAD_SEGMENTS: return "cu_seqlens must start at 0, be non-decreasing and end at total_tokens";
        case MMTRAIN_ERR_UNSUPPORTED: return "unsupported shape";
        case MMTRAIN_ERR_WORKSPACE: return "workspace too small";
        case MMTRAIN_ERR_HIP: return "HIP error";
        case MMTRAIN_ERR_TOO_LARGE: return "input larger than the static scratch of the no-allocation entry point";
        default: return "unknown status";
    }
}

size_t mmtrain_layer_ctx_bytes(const mmtrain_layer_desc *desc, int32_t total_tokens) {
    Dims D;
    if (check_desc(desc, D) != MMTRAIN_OK || total_tokens < 0) return 0;
    Bump b = {nullptr, 0};
    Ctx c;
    carve_ctx(b, D, (size_t)total_tokens, c);
    return ((b.off + 255) & ~size_t(255)) + 256;         // never 0 for a valid description
}

size_t mmtrain_layer_workspace_bytes(const mmtrain_layer_desc *desc, int32_t total_tokens, int32_t n_segments,
                                     int is_bwd) {
    Dims D;
    if (check_desc(desc, D) != MMTRAIN_OK || total_tokens < 0 || n_segments < 0) return 0;
    Bump b = {nullptr, 0};
    if (is_bwd) {
        BwdWs w;
        carve_bwd(b, D, (size_t)total_tokens, w);
    }
    return ((b.off + 255) & ~size_t(255)) + 256;      // never 0 for a valid description
}

int mmtrain_layer_fwd(const mmtrain_layer_desc *desc, const mmtrain_batch *batch, const mmtrain_layer_weights *W,
                      const void *x, void *y, void *ctx, void *workspace, size_t workspace_bytes, void *hip_stream) {
    Dims D;
    int rc = check_desc(desc, D);
    if (rc) return rc;
    if ((rc = check_batch(batch))) return rc;
    if ((rc = check_weights(D, W))) return rc;
    const int T = batch->total_tokens;
    if (T == 0) return MMTRAIN_OK;
    if (!x || !y || !ctx || x == y || misaligned({x, y})) return MMTRAIN_ERR_INVALID_ARG;
    if (((uintptr_t)ctx | (uintptr_t)workspace) & 255) return MMTRAIN_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < mmtrain_layer_workspace_bytes(desc, T, batch->n_segments, 0))
        return MMTRAIN_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)hip_stream;
    const bool enc = D.kind == MMTRAIN_ENCODER;
    Bump b = {(uint8_t *)ctx, 0};
    Ctx c;
    carve_ctx(b, D, (size_t)T, c);

    HIP_TRY(prep_tokens(batch->cu_seqlens_dev, batch->seg_mask_dev, batch->mask_mode, batch->n_segments, T, c.tok_seg,
                        c.tok_info, D.d, D.rope_base, c.rope_cs, st));
    // attention block
    HIP_TRY_TIMED(MMTRAIN_PROF_NORM_FWD, st, norm_fwd(D.dtype, enc, x, W->norm1_w, W->norm1_b, c.h1, c.mean1, c.rstd1, T, D.H, D.eps, st));
    HIP_TRY(gemm(D.dtype, mk(GEMM_NT, T, D.nqkv, D.H, c.h1, D.H, W->w_qkv, D.H, c.qkv, D.nqkv, W->b_qkv), st));
    if (!enc) HIP_TRY_TIMED(MMTRAIN_PROF_ROPE, st, rope_inplace(D.dtype, c.qkv, D.nqkv, T, D.nh + D.nkv, D.d, c.rope_cs, false, st));
    AttnArgs a = mk_attn(D, batch, c);
    {
        ProfScope ps(MMTRAIN_PROF_ATTN_FWD, st);
        HIP_TRY(attn_fwd(D.dtype, a, st));
    }
    HIP_TRY(gemm(D.dtype, mk(GEMM_NT, T, D.H, D.nq, c.o, D.nq, W->w_o, D.nq, c.y1, D.H, W->b_o, x), st));
    // MLP block
    HIP_TRY_TIMED(MMTRAIN_PROF_NORM_FWD, st, norm_fwd(D.dtype, enc, c.y1, W->norm2_w, W->norm2_b, c.h2, c.mean2, c.rstd2, T, D.H, D.eps, st));
    HIP_TRY(gemm(D.dtype, mk(GEMM_NT, T, D.F1, D.H, c.h2, D.H, W->w_fc1, D.H, c.pre, D.F1, W->b_fc1), st));
    if (enc) HIP_TRY_TIMED(MMTRAIN_PROF_ACT_FWD, st, gelu_fwd(D.dtype, c.pre, c.m, (long)T * D.F, st));
    else HIP_TRY_TIMED(MMTRAIN_PROF_ACT_FWD, st, swiglu_fwd(D.dtype, c.pre, c.m, T, D.F, st));
    HIP_TRY(gemm(D.dtype, mk(GEMM_NT, T, D.H, D.F, c.m, D.F, W->w_fc2, D.F, y, D.H, W->b_fc2, c.y1), st));
    return MMTRAIN_OK;
}

int mmtrain_layer_bwd(const mmtrain_layer_desc *desc, const mmtrain_batch *batch, const mmtrain_layer_weights *W,
                      const void *x, const void *dy, const void *ctx, void *dx, const mmtrain_layer_grads *grads,
                      uint32_t flags, void *workspace, size_t workspace_bytes, void *hip_stream) {
    Dims D;
    int rc = check_desc(desc, D);
    if (rc) return rc;
    if ((rc = check_batch(batch))) return rc;
    if ((rc = check_weights(D, W))) return rc;
    if (flags & ~(MMTRAIN_BWD_ACCUMULATE_WGRAD | MMTRAIN_BWD_WGRAD_F32)) return MMTRAIN_ERR_INVALID_ARG;
    if ((rc = check_grads(grads))) return rc;
    const int T = batch->total_tokens;
    const bool accum = flags & MMTRAIN_BWD_ACCUMULATE_WGRAD;
    const bool g32 = flags & MMTRAIN_BWD_WGRAD_F32;          // gradient buffers hold fp32
    const int gdt = g32 ? DT_F32 : D.dtype;                   // dtype of the gradient buffers
    const bool enc = D.kind == MMTRAIN_ENCODER;
    hipStream_t st = (hipStream_t)hip_stream;
    mmtrain_layer_grads G = {};
    if (grads) G = *grads;
    if (T == 0) {                                   // an empty pack contributes zero gradients
        if (!accum) {
            HIP_TRY(fill_zero(G.norm1_w, D.H, gdt, st)); HIP_TRY(fill_zero(G.norm1_b, D.H, gdt, st));
            HIP_TRY(fill_zero(G.w_qkv, (size_t)D.nqkv * D.H, gdt, st)); HIP_TRY(fill_zero(G.b_qkv, D.nqkv, gdt, st));
            HIP_TRY(fill_zero(G.w_o, (size_t)D.H * D.nq, gdt, st)); HIP_TRY(fill_zero(G.b_o, D.H, gdt, st));
            HIP_TRY(fill_zero(G.norm2_w, D.H, gdt, st)); HIP_TRY(fill_zero(G.norm2_b, D.H, gdt, st));
            HIP_TRY(fill_zero(G.w_fc1, (size_t)D.F1 * D.H, gdt, st)); HIP_TRY(fill_zero(G.b_fc1, D.F1, gdt, st));
            HIP_TRY(fill_zero(G.w_fc2, (size_t)D.H * D.F, gdt, st)); HIP_TRY(fill_zero(G.b_fc2, D.H, gdt, st));
        }
        return MMTRAIN_OK;
    }
    if (!x || !dy || !ctx || !dx || misaligned({x, dy, dx})) return MMTRAIN_ERR_INVALID_ARG;
    if (((uintptr_t)ctx | (uintptr_t)workspace) & 255) return MMTRAIN_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < mmtrain_layer_workspace_bytes(desc, T, batch->n_segments, 1))
        return MMTRAIN_ERR_WORKSPACE;
    Bump bc = {(uint8_t *)const_cast<void *>(ctx), 0};
    Ctx c;
    carve_ctx(bc, D, (size_t)T, c);
    Bump bw = {(uint8_t *)workspace, 0};
    BwdWs w;
    carve_bwd(bw, D, (size_t)T, w);
    const int nb = norm_bwd_blocks(T, D.H), ns = colsum_slabs(T);

    // ---- MLP block:  y = y1 + m . Wfc2^T (+ b_fc2)
    HIP_TRY(gemm(D.dtype, splittable(mk(GEMM_NN, T, D.F, D.H, dy, D.H, W->w_fc2, D.F, w.d_m, D.F), w.split_ws, w.split_bytes), st));
    DeferredWgrads later;
    if (G.w_fc2) HIP_TRY(wgrad(D.dtype, splittable(f32out(mk(GEMM_TN, D.H, D.F, T, dy, D.H, c.m, D.F, G.w_fc2, D.F, nullptr, nullptr, accum), g32), w.split_ws, w.split_bytes), later, st));
    // Partial sums (gain, bias and column-sum gradients) are reduced by ONE launch at the end of the pass: every array
    // has a buffer of its own in the workspace.
    ReduceJob jobs[8];
    int n_jobs = 0;
    auto reduce_later = [&](const float *part, void *out, int rows, int N) {
        if (part && out) jobs[n_jobs++] = {part, out, rows, N};
    };
    if (enc && G.b_fc1) {                         // the bias gradient is the column sum of what this kernel writes
        HIP_TRY_TIMED(MMTRAIN_PROF_ACT_BWD, st, gelu_bwd_colsum(D.dtype, w.d_m, c.pre, w.d_pre, T, D.F1, w.part_c, st));
        reduce_later(w.part_c, G.b_fc1, ns, D.F1);
    } else if (enc) HIP_TRY_TIMED(MMTRAIN_PROF_ACT_BWD, st, gelu_bwd(D.dtype, w.d_m, c.pre, w.d_pre, (long)T * D.F, st));
    else HIP_TRY_TIMED(MMTRAIN_PROF_ACT_BWD, st, swiglu_bwd(D.dtype, w.d_m, c.pre, w.d_pre, T, D.F, st));
    HIP_TRY(gemm(D.dtype, splittable(mk(GEMM_NN, T, D.H, D.F1, w.d_pre, D.F1, W->w_fc1, D.H, w.d_h, D.H), w.split_ws, w.split_bytes), st));
    if (G.w_fc1) HIP_TRY(wgrad(D.dtype, splittable(f32out(mk(GEMM_TN, D.F1, D.H, T, w.d_pre, D.F1, c.h2, D.H, G.w_fc1, D.H, nullptr, nullptr, accum), g32), w.split_ws, w.split_bytes), later, st));
    // d_y1 = dy + norm2_bwd(d_h2); the same kernel sums the columns of dy (b_fc2's gradient) and of d_y1 (b_o's)
    HIP_TRY_TIMED(MMTRAIN_PROF_NORM_BWD, st, norm_bwd(D.dtype, enc, w.d_h, c.y1, W->norm2_w, c.mean2, c.rstd2, dy, w.d_y1,
                     G.norm2_w ? w.part_g : nullptr, (enc && G.norm2_b) ? w.part_b : nullptr,
                     (enc && G.b_o) ? w.part_din : nullptr, (enc && G.b_fc2) ? w.part_dres : nullptr, T, D.H, st));
    reduce_later(w.part_g, G.norm2_w, nb, D.H);
    if (enc) {
        reduce_later(w.part_b, G.norm2_b, nb, D.H);
        reduce_later(w.part_din, G.b_o, nb, D.H);
        reduce_later(w.part_dres, G.b_fc2, nb, D.H);
    }

    // ---- attention block:  y1 = x + o . Wo^T (+ b_o)
    HIP_TRY(gemm(D.dtype, splittable(mk(GEMM_NN, T, D.nq, D.H, w.d_y1, D.H, W->w_o, D.nq, w.d_o, D.nq), w.split_ws, w.split_bytes), st));
    if (G.w_o) HIP_TRY(wgrad(D.dtype, splittable(f32out(mk(GEMM_TN, D.H, D.nq, T, w.d_y1, D.H, c.o, D.nq, G.w_o, D.nq, nullptr, nullptr, accum), g32), w.split_ws, w.split_bytes), later, st));
    AttnArgs a = mk_attn(D, batch, c);
    a.d_o = w.d_o; a.d_qkv = w.d_qkv; a.Dsum = w.Dsum;
    const bool fused_unrotate = !enc && D.dtype == DT_BF16 && (D.d == 64 || D.d == 128);       // the matrix-core kernels rotate dQ, dK back themselves
    if (fused_unrotate) a.rope_cs = c.rope_cs;
    {
        ProfScope ps(MMTRAIN_PROF_ATTN_BWD, st);
        HIP_TRY(attn_bwd(D.dtype, a, st));
    }
    if (!enc && !fused_unrotate) HIP_TRY_TIMED(MMTRAIN_PROF_ROPE, st, rope_inplace(D.dtype, w.d_qkv, D.nqkv, T, D.nh + D.nkv, D.d, c.rope_cs, true, st));
    if (enc && G.b_qkv) {
        HIP_TRY(colsum_partials(D.dtype, w.d_qkv, T, D.nqkv, D.nqkv, w.part_c2, st));
        reduce_later(w.part_c2, G.b_qkv, ns, D.nqkv);
    }
    HIP_TRY(gemm(D.dtype, splittable(mk(GEMM_NN, T, D.H, D.nqkv, w.d_qkv, D.nqkv, W->w_qkv, D.H, w.d_h, D.H), w.split_ws, w.split_bytes), st));
    if (G.w_qkv) HIP_TRY(wgrad(D.dtype, splittable(f32out(mk(GEMM_TN, D.nqkv, D.H, T, w.d_qkv, D.nqkv, c.h1, D.H, G.w_qkv, D.H, nullptr, nullptr, accum), g32), w.split_ws, w.split_bytes), later, st));
    // dx = d_y1 + norm1_bwd(d_h1)
    HIP_TRY_TIMED(MMTRAIN_PROF_NORM_BWD, st, norm_bwd(D.dtype, enc, w.d_h, x, W->norm1_w, c.mean1, c.rstd1, w.d_y1, dx,
                     G.norm1_w ? w.part_g1 : nullptr, (enc && G.norm1_b) ? w.part_b1 : nullptr, nullptr, nullptr, T, D.H, st));
    reduce_later(w.part_g1, G.norm1_w, nb, D.H);
    if (enc) reduce_later(w.part_b1, G.norm1_b, nb, D.H);
    HIP_TRY(reduce_jobs(gdt, jobs, n_jobs, accum, st));
    HIP_TRY(run_deferred(later, st));
    return MMTRAIN_OK;
}

// ---- a stack of layers -------------------------------------------------------------
// ctx: the inputs of layers 1 .. n-1 ([T, H] each), then the layer contexts: one per layer, or a single one with
// MMTRAIN_STACK_RECOMPUTE.  Backward workspace: the layer's own, then two [T, H] buffers through which the
// gradient travels down the stack, then (recomputation) one [T, H] buffer for the recomputed layer output.
namespace {
struct StackPlan {
    size_t act, layer_ctx, layer_ws_fwd, layer_ws_bwd;
    bool recompute;
    size_t ctx_bytes(int n) const { return (size_t)(n - 1) * act + (recompute ? 1 : (size_t)n) * layer_ctx; }
    size_t ws_bytes(bool bwd) const { return bwd ? layer_ws_bwd + 2 * act + (recompute ? act : 0) : layer_ws_fwd; }
};
int plan_stack(const mmtrain_layer_desc *desc, int n_layers, int T, int S, uint32_t flags, uint32_t allowed, StackPlan &p) {
    Dims D;
    int rc = check_desc(desc, D);
    if (rc) return rc;
    if (n_layers < 1 || T < 0 || S < 0 || (flags & ~allowed)) return MMTRAIN_ERR_INVALID_ARG;
    p.act = ((size_t)T * D.H * (D.dtype == DT_BF16 ? 2 : 4) + 255) & ~size_t(255);
    p.layer_ctx = mmtrain_layer_ctx_bytes(desc, T);
    p.layer_ws_fwd = mmtrain_layer_workspace_bytes(desc, T, S, 0);
    p.layer_ws_bwd = mmtrain_layer_workspace_bytes(desc, T, S, 1);
    p.recompute = flags & MMTRAIN_STACK_RECOMPUTE;
    return MMTRAIN_OK;
}
}  // namespace

size_t mmtrain_stack_ctx_bytes(const mmtrain_layer_desc *desc, int32_t n_layers, int32_t total_tokens, uint32_t flags) {
    StackPlan p;
    if (plan_stack(desc, n_layers, total_tokens, 0, flags, MMTRAIN_STACK_RECOMPUTE, p)) return 0;
    return p.ctx_bytes(n_layers);
}

size_t mmtrain_stack_workspace_bytes(const mmtrain_layer_desc *desc, int32_t n_layers, int32_t total_tokens,
                                     int32_t n_segments, int is_bwd, uint32_t flags) {
    StackPlan p;
    if (plan_stack(desc, n_layers, total_tokens, n_segments, flags, MMTRAIN_STACK_RECOMPUTE, p)) return 0;
    return p.ws_bytes(is_bwd != 0);
}

int mmtrain_stack_fwd(const mmtrain_layer_desc *desc, int32_t n_layers, const mmtrain_batch *batch,
                      const mmtrain_layer_weights *weights, const void *x, void *y, void *ctx, uint32_t flags,
                      void *workspace, size_t workspace_bytes, void *hip_stream) {
    Dims D;
    int rc = check_desc(desc, D);
    if (rc) return rc;
    if ((rc = check_batch(batch))) return rc;
    StackPlan p;
    if ((rc = plan_stack(desc, n_layers, batch->total_tokens, batch->n_segments, flags, MMTRAIN_STACK_RECOMPUTE, p))) return rc;
    if (!weights) return MMTRAIN_ERR_INVALID_ARG;
    for (int l = 0; l < n_layers; ++l)
        if ((rc = check_weights(D, &weights[l]))) return rc;
    if (batch->total_tokens == 0) return MMTRAIN_OK;
    if (!x || !y || !ctx || x == y || misaligned({x, y}) || (((uintptr_t)ctx | (uintptr_t)workspace) & 255)) return MMTRAIN_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < p.ws_bytes(false)) return MMTRAIN_ERR_WORKSPACE;
    uint8_t *acts = (uint8_t *)ctx, *ctxs = acts + (size_t)(n_layers - 1) * p.act;
    for (int l = 0; l < n_layers; ++l) {
        const void *in = l == 0 ? x : acts + (size_t)(l - 1) * p.act;
        void *out = l == n_layers - 1 ? y : acts + (size_t)l * p.act;
        void *lctx = ctxs + (p.recompute ? 0 : (size_t)l * p.layer_ctx);
        if ((rc = mmtrain_layer_fwd(desc, batch, &weights[l], in, out, lctx, workspace, workspace_bytes, hip_stream))) return rc;
    }
    return MMTRAIN_OK;
}

int mmtrain_stack_bwd(const mmtrain_layer_desc *desc, int32_t n_layers, const mmtrain_batch *batch,
                      const mmtrain_layer_weights *weights, const void *x, const void *dy, void *ctx, void *dx,
                      const mmtrain_layer_grads *grads, uint32_t flags, void *workspace, size_t workspace_bytes,
                      void *hip_stream) {
    Dims D;
    int rc = check_desc(desc, D);
    if (rc) return rc;
    if ((rc = check_batch(batch))) return rc;
    StackPlan p;
    const uint32_t bwd_flags = MMTRAIN_BWD_ACCUMULATE_WGRAD | MMTRAIN_BWD_WGRAD_F32;
    if ((rc = plan_stack(desc, n_layers, batch->total_tokens, batch->n_segments, flags, MMTRAIN_STACK_RECOMPUTE | bwd_flags, p)))
        return rc;
    if (!weights) return MMTRAIN_ERR_INVALID_ARG;
    for (int l = 0; l < n_layers; ++l) {
        if ((rc = check_weights(D, &weights[l]))) return rc;
        if (grads && (rc = check_grads(&grads[l]))) return rc;
    }
    const uint32_t lflags = flags & bwd_flags;
    if (batch->total_tokens == 0) {                 // an empty pack: every layer's gradients are zero (or left as they are)
        for (int l = 0; l < n_layers; ++l)
            if ((rc = mmtrain_layer_bwd(desc, batch, &weights[l], x, dy, ctx, dx, grads ? &grads[l] : nullptr, lflags, workspace,
                                        workspace_bytes, hip_stream))) return rc;
        return MMTRAIN_OK;
    }
    if (!x || !dy || !ctx || !dx || misaligned({x, dy, dx}) || (((uintptr_t)ctx | (uintptr_t)workspace) & 255)) return MMTRAIN_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < p.ws_bytes(true)) return MMTRAIN_ERR_WORKSPACE;
    uint8_t *acts = (uint8_t *)ctx, *ctxs = acts + (size_t)(n_layers - 1) * p.act;
    uint8_t *ws = (uint8_t *)workspace;
    uint8_t *grad_buf[2] = {ws + p.layer_ws_bwd, ws + p.layer_ws_bwd + p.act};
    uint8_t *y_again = ws + p.layer_ws_bwd + 2 * p.act;
    const void *g_in = dy;
    for (int l = n_layers - 1; l >= 0; --l) {
        const void *in = l == 0 ? x : acts + (size_t)(l - 1) * p.act;
        void *lctx = ctxs + (p.recompute ? 0 : (size_t)l * p.layer_ctx);
        if (p.recompute && l != n_layers - 1)
            if ((rc = mmtrain_layer_fwd(desc, batch, &weights[l], in, y_again, lctx, workspace, p.layer_ws_bwd, hip_stream))) return rc;
        void *g_out = l == 0 ? dx : (void *)grad_buf[l & 1];
        if ((rc = mmtrain_layer_bwd(desc, batch, &weights[l], in, g_in, lctx, g_out, grads ? &grads[l] : nullptr, lflags,
                                    workspace, p.layer_ws_bwd, hip_stream))) return rc;
        g_in = g_out;
    }
    return MMTRAIN_OK;
}

// ---- profiling ---------------------------------------------------------------------

void mmtrain_profile_gemm_clock(void *device_counters) { g_gemm_clock = (unsigned long long *)device_counters; }

void mmtrain_profile_attn_busy(void *device_counters) { g_attn_busy = (unsigned long long *)device_counters; }

void mmtrain_profile_enable(int class_mask) { g_prof.mask = class_mask & MMTRAIN_PROF_ALL; }

int mmtrain_profile_read(int32_t kind, double *total_ms, int64_t *launches, int reset) {
    if (!total_ms || !launches) return MMTRAIN_ERR_INVALID_ARG;
    double ms = 0.0;
    int64_t n = 0;
    for (auto &s : g_prof.spans) {
        if (s.kind != kind) continue;
        if (hipEventSynchronize(s.b) != hipSuccess) return MMTRAIN_ERR_HIP;
        float t = 0.f;
        if (hipEventElapsedTime(&t, s.a, s.b) != hipSuccess) return MMTRAIN_ERR_HIP;
        ms += t; ++n;
    }
    *total_ms = ms; *launches = n;
    if (reset) {
        std::vector<Profiler::Span> keep;
        for (auto &s : g_prof.spans) {
            if (s.kind == kind) { g_prof.pool.push_back(s.a); g_prof.pool.push_back(s.b); }
            else keep.push_back(s);
        }
        g_prof.spans.swap(keep);
    }
    return MMTRAIN_OK;
}

// ---- operator-level entry points ----------------------------------------------------

int mmtrain_gemm(int32_t dtype, int32_t layout, int32_t M, int32_t N, int32_t K, const void *A, int32_t lda,
                 const void *B, int32_t ldb, void *C, int32_t ldc, const void *bias, const void *residual,
                 uint32_t flags, void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (dtype != MMTRAIN_F32 && dtype != MMTRAIN_BF16) return MMTRAIN_ERR_INVALID_ARG;
    if (layout < MMTRAIN_GEMM_NT || layout > MMTRAIN_GEMM_TN) return MMTRAIN_ERR_INVALID_ARG;
    if (M < 0 || N < 0 || K < 0 || (flags & ~MMTRAIN_GEMM_ACCUMULATE)) return MMTRAIN_ERR_INVALID_ARG;
    if (M == 0 || N == 0) return MMTRAIN_OK;
    if (!C || (K > 0 && (!A || !B))) return MMTRAIN_ERR_INVALID_ARG;
    const int min_lda = layout == MMTRAIN_GEMM_TN ? M : K, min_ldb = layout == MMTRAIN_GEMM_NT ? K : N;
    if (lda < min_lda || ldb < min_ldb || ldc < N) return MMTRAIN_ERR_INVALID_ARG;
    if ((workspace_bytes && !workspace) || ((uintptr_t)workspace & 255)) return MMTRAIN_ERR_INVALID_ARG;
    GemmArgs g = mk(layout, M, N, K, A, lda, B, ldb, C, ldc, bias, residual, flags & MMTRAIN_GEMM_ACCUMULATE);
    if (workspace_bytes) g = splittable(g, workspace, workspace_bytes);
    if (dtype == MMTRAIN_BF16 && !gemm_mfma_supported(g) && K > 0) return MMTRAIN_ERR_UNSUPPORTED;
    HIP_TRY(gemm(dtype, g, (hipStream_t)hip_stream));
    return MMTRAIN_OK;
}

size_t mmtrain_gemm_workspace_bytes(int32_t layout, int32_t M, int32_t N) {
    if (M <= 0 || N <= 0 || (layout != MMTRAIN_GEMM_NN && layout != MMTRAIN_GEMM_TN)) return 0;
    const size_t tiles = (((size_t)M + 255) / 256) * (((size_t)N + 255) / 256);
    if (layout == MMTRAIN_GEMM_NN && tiles <= 128) return 0;       // only weight gradients are cut when tiles are few
    return gemm_scratch_bytes((size_t)M, (size_t)N);
}

size_t mmtrain_attn_workspace_bytes(int32_t total_tokens, int32_t n_segments, int32_t n_heads) {
    if (total_tokens < 0 || n_segments < 0 || n_heads <= 0) return 0;
    Bump b = {nullptr, 0};
    b.take<int>((size_t)total_tokens);
    b.take<int2>((size_t)total_tokens);
    b.take<float>((size_t)total_tokens * n_heads);
    return ((b.off + 255) & ~size_t(255)) + 256;
}

// `tensors`: the call's device tensors, all required and 16-byte aligned (checked before anything is enqueued)
static int attn_common(const mmtrain_layer_desc *desc, const mmtrain_batch *batch, Dims &D, void *workspace,
                       size_t workspace_bytes, std::initializer_list<const void *> tensors, AttnArgs &a, hipStream_t st) {
    int rc = check_desc(desc, D);
    if (rc) return rc;
    if ((rc = check_batch(batch))) return rc;
    const int T = batch->total_tokens;
    if (T == 0) return MMTRAIN_OK;
    for (const void *p : tensors)
        if (!p) return MMTRAIN_ERR_INVALID_ARG;
    if (misaligned(tensors)) return MMTRAIN_ERR_INVALID_ARG;
    if ((uintptr_t)workspace & 255) return MMTRAIN_ERR_INVALID_ARG;
    if (!workspace || workspace_bytes < mmtrain_attn_workspace_bytes(T, batch->n_segments, D.nh))
        return MMTRAIN_ERR_WORKSPACE;
    Bump b = {(uint8_t *)workspace, 0};
    int *tok_seg = b.take<int>((size_t)T);
    int2 *tok_info = b.take<int2>((size_t)T);
    float *Dsum = b.take<float>((size_t)T * D.nh);
    a = AttnArgs{};
    a.T = T; a.S = batch->n_segments; a.nh = D.nh; a.nkv = D.nkv; a.d = D.d; a.scale = D.scale;
    a.cu = batch->cu_seqlens_dev; a.modes = batch->seg_mask_dev; a.default_mode = batch->mask_mode;
    a.tok_seg = tok_seg; a.tok_info = tok_info; a.ld_qkv = D.nqkv; a.Dsum = Dsum;
    a.cu_busy = g_attn_busy;
    attn_tile_order(batch->cu_seqlens_host, batch->seg_mask_host, batch->mask_mode, batch->n_segments, T, a);
    HIP_TRY(prep_tokens(batch->cu_seqlens_dev, batch->seg_mask_dev, batch->mask_mode, batch->n_segments, T, tok_seg, tok_info,
                        D.d, 0.f, nullptr, st));
    return MMTRAIN_OK;
}

int mmtrain_attn_fwd(const mmtrain_layer_desc *desc, const mmtrain_batch *batch, const void *qkv, void *o,
                     float *lse, void *workspace, size_t workspace_bytes, void *hip_stream) {
    Dims D;
    AttnArgs a;
    hipStream_t st = (hipStream_t)hip_stream;
    int rc = attn_common(desc, batch, D, workspace, workspace_bytes, {qkv, o, lse}, a, st);
    if (rc || batch->total_tokens == 0) return rc;
    a.qkv = qkv; a.o = o; a.lse = lse;
    HIP_TRY(attn_fwd(D.dtype, a, st));
    return MMTRAIN_OK;
}

int mmtrain_attn_bwd(const mmtrain_layer_desc *desc, const mmtrain_batch *batch, const void *qkv, const void *o,
                     const float *lse, const void *d_o, void *d_qkv, void *workspace, size_t workspace_bytes,
                     void *hip_stream) {
    Dims D;
    AttnArgs a;
    hipStream_t st = (hipStream_t)hip_stream;
    int rc = attn_common(desc, batch, D, workspace, workspace_bytes, {qkv, o, lse, d_o, d_qkv}, a, st);
    if (rc || batch->total_tokens == 0) return rc;
    a.qkv = qkv; a.o = const_cast<void *>(o); a.lse = const_cast<float *>(lse); a.d_o = d_o; a.d_qkv = d_qkv;
    HIP_TRY(attn_bwd(D.dtype, a, st));
    return MMTRAIN_OK;
}

// ---- attention backward for callers that cannot allocate ---------------------------------------------------
// The scratch mmtrain_attn_bwd takes as its workspace (per-token segment tables, D = rowsum(dO * O) per head and
// token, handed from the dQ kernel to the dK/dV kernel) lives in a file-scope device array instead.  In host code
// the array's name is only a stand-in: its device address is looked up once per device and used from then on.
}  // extern "C"

static __device__ __align__(256) unsigned char scratch[MMTRAIN_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};           // device address of `scratch` on each device, once looked up

// The current device's copy of the array (every device holds its own, at its own address).
int scratch_address(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return MMTRAIN_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return MMTRAIN_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return MMTRAIN_OK;
}
}  // namespace

extern "C" {

int mmtrain_attn_bwd_noalloc(const mmtrain_layer_desc *desc, const mmtrain_batch *batch, const void *qkv, const void *o,
                             const float *lse, const void *d_o, void *d_qkv, void *hip_stream) {
    Dims D;
    int rc = check_desc(desc, D);
    if (rc) return rc;
    if ((rc = check_batch(batch))) return rc;
    if (batch->total_tokens > MMTRAIN_NOALLOC_MAX_TOKENS ||
        (int64_t)batch->total_tokens * D.nh > MMTRAIN_NOALLOC_MAX_HEAD_TOKENS ||
        mmtrain_attn_workspace_bytes(batch->total_tokens, batch->n_segments, D.nh) > MMTRAIN_NOALLOC_SCRATCH_BYTES)
        return MMTRAIN_ERR_TOO_LARGE;
    if (batch->total_tokens == 0) return MMTRAIN_OK;
    if (!qkv || !o || !lse || !d_o || !d_qkv) return MMTRAIN_ERR_INVALID_ARG;
    void *ws = nullptr;
    if ((rc = scratch_address(&ws))) return rc;
    // Nothing in the scratch has to start at zero: the kernels write every entry they later read.
    return mmtrain_attn_bwd(desc, batch, qkv, o, lse, d_o, d_qkv, ws, MMTRAIN_NOALLOC_SCRATCH_BYTES, hip_stream);
}

int mmtrain_intra_reorder(const double *sizes, int32_t n, int32_t m, int32_t *order, int32_t *group_begin,
                          double *group_load) {
    if (n < 0 || m <= 0 || (n > 0 && (!sizes || !order))) return MMTRAIN_ERR_INVALID_ARG;
    for (int32_t i = 0; i < n; ++i)
        if (!(sizes[i] >= 0.0) || sizes[i] > 1e300) return MMTRAIN_ERR_INVALID_ARG;     // also rejects NaN
    intra_reorder(sizes, n, m, order, group_begin, group_load);
    return MMTRAIN_OK;
}

static bool durations_ok(const double *v, size_t n) {
    for (size_t i = 0; i < n; ++i)
        if (!(v[i] >= 0.0) || v[i] > 1e300) return false;              // also rejects NaN
    return true;
}

int mmtrain_pipeline_1f1b(const double *fwd, const double *bwd, int32_t p, int32_t l, const int32_t *order,
                          double *makespan, double *intervals) {
    if (p < 1 || l < 0 || (l > 0 && (!fwd || !bwd))) return MMTRAIN_ERR_INVALID_ARG;
    if ((size_t)p * (size_t)l > (size_t)1 << 28) return MMTRAIN_ERR_INVALID_ARG;
    if (!durations_ok(fwd, (size_t)p * l) || !durations_ok(bwd, (size_t)p * l)) return MMTRAIN_ERR_INVALID_ARG;
    if (order) {
        std::vector<char> seen((size_t)l, 0);
        for (int32_t q = 0; q < l; ++q) {
            if (order[q] < 0 || order[q] >= l || seen[order[q]]) return MMTRAIN_ERR_INVALID_ARG;
            seen[order[q]] = 1;
        }
    }
    if (l == 0) { if (makespan) *makespan = 0.0; return MMTRAIN_OK; }
    return pipeline_1f1b(fwd, bwd, p, l, order, makespan, intervals) ? MMTRAIN_ERR_INVALID_ARG : MMTRAIN_OK;
}

int mmtrain_inter_reorder(const double *fwd, const double *bwd, int32_t p, int32_t l, const double *sizes, int32_t *order,
                          double *intervals_seen, int32_t *n_intervals) {
    if (p < 1 || l < 0 || (l > 0 && (!fwd || !bwd || !order))) return MMTRAIN_ERR_INVALID_ARG;
    if ((size_t)p * (size_t)l > (size_t)1 << 28) return MMTRAIN_ERR_INVALID_ARG;
    if (!durations_ok(fwd, (size_t)p * l) || !durations_ok(bwd, (size_t)p * l)) return MMTRAIN_ERR_INVALID_ARG;
    if (sizes && !durations_ok(sizes, (size_t)l)) return MMTRAIN_ERR_INVALID_ARG;
    inter_reorder(fwd, bwd, p, l, sizes, order, intervals_seen, n_intervals);
    return MMTRAIN_OK;
}

int mmtrain_adam_step(const mmtrain_adam_desc *d, int64_t n, float *master, float *grad, float *exp_avg,
                      float *exp_avg_sq, void *param_out, int32_t param_dtype, void *hip_stream) {
    if (!d || d->struct_size != sizeof(mmtrain_adam_desc) || n < 0) return MMTRAIN_ERR_INVALID_ARG;
    if (param_dtype != MMTRAIN_F32 && param_dtype != MMTRAIN_BF16) return MMTRAIN_ERR_INVALID_ARG;
    if (!(d->lr >= 0.f) || !(d->beta1 >= 0.f && d->beta1 < 1.f) || !(d->beta2 >= 0.f && d->beta2 < 1.f) || !(d->eps > 0.f) ||
        !(d->weight_decay >= 0.f) || !(d->grad_scale == d->grad_scale) || d->step < 1)
        return MMTRAIN_ERR_INVALID_ARG;
    if (n == 0) return MMTRAIN_OK;
    if (!master || !grad || !exp_avg || !exp_avg_sq) return MMTRAIN_ERR_INVALID_ARG;
    if (((uintptr_t)master | (uintptr_t)grad | (uintptr_t)exp_avg | (uintptr_t)exp_avg_sq | (uintptr_t)param_out) & 15)
        return MMTRAIN_ERR_INVALID_ARG;
    AdamArgs a;
    a.lr = d->lr; a.beta1 = d->beta1; a.beta2 = d->beta2; a.eps = d->eps; a.weight_decay = d->weight_decay;
    a.grad_scale = d->grad_scale;
    // 1 - beta and the bias corrections in double on the host: in fp32, 1 - 0.999 is off by 5e-5 and 1 - beta^t
    // loses most of its digits for small t
    a.omb1 = (float)(1.0 - (double)d->beta1); a.omb2 = (float)(1.0 - (double)d->beta2);
    a.inv_bias1 = (float)(1.0 / (1.0 - pow((double)d->beta1, (double)d->step)));
    a.inv_bias2 = (float)(1.0 / (1.0 - pow((double)d->beta2, (double)d->step)));
    a.zero_grad = d->zero_grad ? 1 : 0;
    HIP_TRY(adam_step(param_dtype, (size_t)n, master, grad, exp_avg, exp_avg_sq, param_out, a, (hipStream_t)hip_stream));
    return MMTRAIN_OK;
}

}  // extern "C"
