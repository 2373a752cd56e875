/*
 * mmtrain -- forward and backward of one transformer layer over a packed
 * multimodal microbatch, for AMD MI355X (gfx950).
 *
 * The paper trains multimodal LLMs whose per-GPU work is a stack of identical
 * transformer layers (Section 2.2 "Model Heterogeneity"; Section 4.2, where the
 * LLM backbone is described as homogeneous transformer layers; Table 2 for the
 * Llama3 shapes; Section 7 "Models" for the ViT encoder) applied to fixed-length
 * sequences that interleave text subsequences and image subsequences
 * (Section 2.1, Section 2.3 "Data Heterogeneity", Section 7 "Datasets").  It
 * treats the layer as a black box; this library is that black box: one GPU's
 * share of a training step.
 *
 * Layer kinds
 *   DECODER  y1 = x + Wo.attn(rope(Wqkv.rmsnorm1(x)));  y = y1 + Wfc2.(silu(g)*u),
 *            [g | u] = Wfc1.rmsnorm2(y1).   No biases.  Grouped-query attention
 *            (query head h reads key/value head h / (n_heads / n_kv_heads)).
 *            Rotary embedding pairs feature i with i + head_dim/2; positions
 *            restart at 0 in every segment.
 *   ENCODER  same skeleton with LayerNorm (gain + bias), biases on all four
 *            linears, no rotary embedding, y = y1 + Wfc2.gelu_erf(Wfc1.ln2(y1)+b)+b.
 *
 * Packing.  T tokens are stored back to back in segment order; cu_seqlens[S+1]
 * (cu[0] = 0, cu[S] = T, non-decreasing; empty segments allowed) cuts them into
 * S segments.  Attention never crosses a segment boundary; inside a segment it
 * is causal (key j <= query i) or bidirectional.
 *
 * Layout.  Activations are row-major [T, features].  Weights are row-major
 * [out_features, in_features].  Every gradient has the shape and dtype of what
 * it differentiates.  dtype is the storage type of all activations, weights and
 * gradients: MMTRAIN_BF16 (bf16 storage, fp32 accumulation, MFMA kernels) or
 * MMTRAIN_F32 (fp32 storage and arithmetic).
 *
 * Ownership.  The library never allocates, frees or retains memory.  The caller
 * owns x, y, dy, dx, weights, gradients, `ctx` (opaque; written by fwd, read by
 * bwd; size from mmtrain_layer_ctx_bytes) and `workspace` (scratch; size from
 * mmtrain_layer_workspace_bytes; may be reused by later calls on the same
 * stream).  All of these are DEVICE pointers unless a field says "host"; ctx and
 * workspace must be 256-byte aligned and every tensor (x, y, dy, dx, weights,
 * gradients, qkv, o, lse ...) at least 16-byte aligned -- the kernels move 16 bytes
 * per lane -- else MMTRAIN_ERR_INVALID_ARG.  Host arrays need only stay valid
 * during the call.
 *
 * Asynchrony.  Calls validate on the host, enqueue kernels on `hip_stream`
 * (a hipStream_t; NULL = the default stream) and return without synchronising.
 *
 * Threads and devices.  The library is written for one GPU per process (the
 * device that is current at the first call).  Calls may come from several host
 * threads on different streams as long as each has its own ctx and workspace:
 * what the library sets up at first use (kernel attributes, the device's unit
 * counts, a per-thread cache of the attention tile order) is idempotent.  The
 * measurement aids (mmtrain_profile_*) are process-wide and not thread-safe;
 * mmtrain_attn_bwd_noalloc shares one scratch array per device.
 *
 * Errors.  Every call returns an mmtrain_status (0 = OK, negative = error).
 * Argument and segment validation happens before any HIP call; on such an error
 * nothing has been enqueued.  The library never throws and never aborts.
 */
#ifndef MMTRAIN_H
#define MMTRAIN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MMTRAIN_API __attribute__((visibility("default")))

typedef enum {
    MMTRAIN_OK = 0,
    MMTRAIN_ERR_INVALID_ARG = -1,   /* NULL where a pointer is required, bad enum, bad struct_size   */
    MMTRAIN_ERR_BAD_SEGMENTS = -2,  /* cu_seqlens not starting at 0, decreasing, or not ending at T  */
    MMTRAIN_ERR_UNSUPPORTED = -3,   /* shape outside the supported set (see mmtrain_layer_desc)      */
    MMTRAIN_ERR_WORKSPACE = -4,     /* workspace_bytes smaller than mmtrain_layer_workspace_bytes    */
    MMTRAIN_ERR_HIP = -5,           /* a HIP call or kernel launch reported an error                 */
    MMTRAIN_ERR_TOO_LARGE = -6      /* input beyond the fixed maximum of mmtrain_attn_bwd_noalloc    */
} mmtrain_status;

typedef enum { MMTRAIN_F32 = 0, MMTRAIN_BF16 = 1 } mmtrain_dtype;
typedef enum { MMTRAIN_DECODER = 0, MMTRAIN_ENCODER = 1 } mmtrain_layer_kind;
typedef enum {
    MMTRAIN_MASK_CAUSAL = 0,        /* key j <= query i, same segment */
    MMTRAIN_MASK_BIDIR = 1          /* every key of the same segment  */
} mmtrain_mask_mode;

/* Layer description.  Supported: head_dim in {64, 128}, and with bf16 storage also every other multiple of
 * 16 below 128 (80 is the ViT-Huge head; such heads are zero-padded to 64 or 128 inside the kernels); n_heads % n_kv_heads == 0
 * (encoder: n_kv_heads == n_heads); hidden, ffn_hidden and n_heads*head_dim
 * multiples of 16.  Anything else: MMTRAIN_ERR_UNSUPPORTED. */
typedef struct {
    uint32_t struct_size;           /* sizeof(mmtrain_layer_desc) */
    int32_t kind;                   /* mmtrain_layer_kind */
    int32_t dtype;                  /* mmtrain_dtype */
    int32_t hidden;                 /* H */
    int32_t n_heads;                /* nh */
    int32_t n_kv_heads;             /* nkv */
    int32_t head_dim;               /* d */
    int32_t ffn_hidden;             /* F */
    float norm_eps;
    float rope_base;                /* decoder only */
    float softmax_scale;            /* 0 => 1/sqrt(head_dim) */
} mmtrain_layer_desc;

/* One packed microbatch (Section 2.3: a sequence of interleaved subsequences). */
typedef struct {
    int32_t total_tokens;           /* T >= 0 */
    int32_t n_segments;             /* S >= 0 */
    const int32_t *cu_seqlens_dev;  /* device [S+1] */
    const int32_t *cu_seqlens_host; /* host   [S+1], same values: validation and launch sizing */
    int32_t mask_mode;              /* mmtrain_mask_mode for every segment unless seg_mask_* given */
    const uint8_t *seg_mask_dev;    /* optional device [S]: per-segment mmtrain_mask_mode */
    const uint8_t *seg_mask_host;   /* optional host   [S]: same values; both or neither */
} mmtrain_batch;

/* Parameters.  *_b and b_* are NULL for the decoder. */
typedef struct {
    const void *norm1_w, *norm1_b;  /* [H] */
    const void *w_qkv, *b_qkv;      /* [(nh + 2 nkv) d, H]; rows: q heads | k heads | v heads */
    const void *w_o, *b_o;          /* [H, nh d] */
    const void *norm2_w, *norm2_b;  /* [H] */
    const void *w_fc1, *b_fc1;      /* decoder [2F, H]: gate rows then up rows; encoder [F, H] */
    const void *w_fc2, *b_fc2;      /* [H, F] */
} mmtrain_layer_weights;

/* Where to write parameter gradients.  A NULL member means "do not compute this
 * gradient" -- the frozen-module case of Section 7.3, where a frozen module runs
 * forward and propagates input gradients but computes no weight gradients. */
typedef struct {
    void *norm1_w, *norm1_b, *w_qkv, *b_qkv, *w_o, *b_o;
    void *norm2_w, *norm2_b, *w_fc1, *b_fc1, *w_fc2, *b_fc2;
} mmtrain_layer_grads;

/* Gradient accumulation over microbatches (summation is commutative, the
 * property Section 5.2 relies on for reordering): matrix and bias and gain
 * gradients are added to the buffers' contents instead of overwriting them. */
#define MMTRAIN_BWD_ACCUMULATE_WGRAD 1u
/* fp32 main-gradient buffers: every non-NULL member of mmtrain_layer_grads points to fp32 storage of the
 * parameter's shape, whatever desc->dtype is (mixed-precision training, Section 3, keeps the accumulated
 * gradients of bf16 parameters in fp32).  The products are accumulated in fp32 as always and are then
 * written, or added with MMTRAIN_BWD_ACCUMULATE_WGRAD, without the rounding to the storage dtype. */
#define MMTRAIN_BWD_WGRAD_F32 2u

/* Bytes of `ctx` for a pack of total_tokens tokens.  0 on invalid desc. */
MMTRAIN_API size_t mmtrain_layer_ctx_bytes(const mmtrain_layer_desc *desc, int32_t total_tokens);

/* Bytes of `workspace` for fwd (is_bwd = 0) or bwd (is_bwd = 1).  0 on invalid desc. */
MMTRAIN_API size_t mmtrain_layer_workspace_bytes(const mmtrain_layer_desc *desc, int32_t total_tokens,
                                     int32_t n_segments, int is_bwd);

/* Forward:  y[T,H] = layer(x[T,H]).  Fills ctx.  x and y may not alias. */
MMTRAIN_API int mmtrain_layer_fwd(const mmtrain_layer_desc *desc, const mmtrain_batch *batch,
                      const mmtrain_layer_weights *weights, const void *x, void *y, void *ctx,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/* Backward:  given dy[T,H] and the ctx of the matching forward call, writes dx[T,H]
 * and every non-NULL member of grads (grads itself may be NULL: input gradient only). */
MMTRAIN_API int mmtrain_layer_bwd(const mmtrain_layer_desc *desc, const mmtrain_batch *batch,
                      const mmtrain_layer_weights *weights, const void *x, const void *dy,
                      const void *ctx, void *dx, const mmtrain_layer_grads *grads, uint32_t flags,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/* ------------------------------------------------------------------------
 * A stack of n_layers layers of one description applied in sequence (the
 * homogeneous transformer layers of Section 4.2; Table 2 lists the depths):
 * y = layer[n-1](... layer[0](x)).  `weights` (and `grads`, which may be NULL,
 * as may any of its members' members) are HOST arrays of n_layers structures
 * holding device pointers.  `ctx` is opaque as for one layer.
 *
 * Without flags the stack keeps every layer's context for the backward pass.
 * With MMTRAIN_STACK_RECOMPUTE (pass the same flag to all four calls) forward
 * keeps only the input of every layer ([T, hidden] each) plus one layer
 * context; backward runs each layer's forward again right before its
 * backward (the last layer's context is still there from the forward pass).
 * The kernels are deterministic, so both modes give bit-identical results;
 * recomputation trades one extra forward pass for n_layers - 1 contexts of
 * memory.  mmtrain_stack_bwd takes the MMTRAIN_BWD_* flags as well.
 * ------------------------------------------------------------------------ */
#define MMTRAIN_STACK_RECOMPUTE 256u

MMTRAIN_API size_t mmtrain_stack_ctx_bytes(const mmtrain_layer_desc *desc, int32_t n_layers, int32_t total_tokens,
                                           uint32_t flags);
MMTRAIN_API size_t mmtrain_stack_workspace_bytes(const mmtrain_layer_desc *desc, int32_t n_layers,
                                                 int32_t total_tokens, int32_t n_segments, int is_bwd,
                                                 uint32_t flags);
MMTRAIN_API int mmtrain_stack_fwd(const mmtrain_layer_desc *desc, int32_t n_layers, const mmtrain_batch *batch,
                                  const mmtrain_layer_weights *weights, const void *x, void *y, void *ctx,
                                  uint32_t flags, void *workspace, size_t workspace_bytes, void *hip_stream);
MMTRAIN_API int mmtrain_stack_bwd(const mmtrain_layer_desc *desc, int32_t n_layers, const mmtrain_batch *batch,
                                  const mmtrain_layer_weights *weights, const void *x, const void *dy,
                                  void *ctx, void *dx, const mmtrain_layer_grads *grads, uint32_t flags,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);

MMTRAIN_API const char *mmtrain_status_string(int status);

/* ------------------------------------------------------------------------
 * Measurement aid (not part of the layer's arithmetic).  While enabled, the
 * layer calls bracket each launch of the enabled classes below with HIP events
 * on the caller's stream; mmtrain_profile_read waits for the recorded events of
 * one class, returns their summed duration and count, and (reset != 0) forgets
 * them.  mmtrain_profile_enable takes a mask: bit k enables class k, 0 switches
 * everything off, MMTRAIN_PROF_ALL enables all (an event pair costs a few
 * microseconds on the stream, so a timed region enables only what it reports).
 * Process-wide, not thread-safe; event objects are created on demand and
 * reused.  Used by the benchmark to obtain per-kernel launch durations inside
 * the timed region.
 * ------------------------------------------------------------------------ */
typedef enum {
    MMTRAIN_PROF_GEMM_NT = 0, MMTRAIN_PROF_GEMM_NN = 1, MMTRAIN_PROF_GEMM_TN = 2,
    MMTRAIN_PROF_ATTN_FWD = 3, MMTRAIN_PROF_ATTN_BWD = 4,
    /* the memory-bound kernels: normalisation forward / backward, rotary embedding, SwiGLU or GELU forward / backward */
    MMTRAIN_PROF_NORM_FWD = 5, MMTRAIN_PROF_NORM_BWD = 6, MMTRAIN_PROF_ROPE = 7,
    MMTRAIN_PROF_ACT_FWD = 8, MMTRAIN_PROF_ACT_BWD = 9
} mmtrain_prof_kind;
#define MMTRAIN_PROF_ALL 0x3ff
MMTRAIN_API void mmtrain_profile_enable(int class_mask);
MMTRAIN_API int mmtrain_profile_read(int32_t kind, double *total_ms, int64_t *launches, int reset);
/* Load balance of the attention kernels over the compute units (measurement aid; bf16 storage only).  While
 * device_counters is not NULL, every workgroup of the attention kernels adds its run time, in ticks of the GPU's
 * constant 100 MHz counter, to the entry of the compute unit it ran on: device memory, uint64[3][1024], rows =
 * forward, dQ, dK/dV; the entry index is the hardware's compute-unit identifier (XCD, shader engine, unit), so most
 * of the 1024 entries stay untouched.  The caller zeroes the buffer, owns it and keeps it alive until it has
 * passed NULL again and the stream has drained.  Process-wide, not thread-safe. */
MMTRAIN_API void mmtrain_profile_attn_busy(void *device_counters);
/* Shader clock under the bf16 GEMM kernel (measurement aid).  While device_counters (device memory, uint64[4]) is not
 * NULL, the first workgroup of every matrix-core GEMM launch stores the shader-clock counter and the GPU's constant
 * 100 MHz counter at its start ([0], [1]) and at its end ([2], [3]); ([2] - [0]) / ([3] - [1]) x 100 MHz is the clock the
 * compute unit sustained during that launch (the last launch's values remain).  Same ownership rules as above. */
MMTRAIN_API void mmtrain_profile_gemm_clock(void *device_counters);

/* ------------------------------------------------------------------------
 * Operator-level entry points: the kernels the layer calls are built from,
 * exposed one by one so that each can be tested and timed on its own.  Same
 * conventions as above (device pointers, caller-owned, asynchronous).
 * ------------------------------------------------------------------------ */

typedef enum {
    MMTRAIN_GEMM_NT = 0,            /* C[M,N] = A[M,K] . B[N,K]^T   (linear forward)   */
    MMTRAIN_GEMM_NN = 1,            /* C[M,N] = A[M,K] . B[K,N]     (input gradient)   */
    MMTRAIN_GEMM_TN = 2             /* C[M,N] = A[K,M]^T . B[K,N]   (weight gradient)  */
} mmtrain_gemm_layout;

#define MMTRAIN_GEMM_ACCUMULATE 1u  /* C += instead of C =  */

/* C = op(A).op(B) (+ bias[N] broadcast over rows) (+ residual[M,N], leading dimension ldc).
 * Row-major with leading dimensions lda/ldb/ldc in elements.  fp32 accumulation.
 * bf16: K-contiguous operands need K % 8 == 0, strided ones N (or M) % 8 == 0, and
 * lda, ldb, ldc multiples of 8; otherwise MMTRAIN_ERR_UNSUPPORTED.
 * workspace (device memory, 256-byte aligned, caller-owned, may be NULL with 0 bytes) is
 * scratch for fp32 partial products.  With it, a bf16 NN or TN product without bias or
 * residual may be cut along K where that fills the chip better: a weight gradient whose
 * output has few 256 x 256 tiles, or the partly filled last round of tiles of a large
 * product.  mmtrain_gemm_workspace_bytes() returns a size that allows every such cut; a
 * smaller workspace only restricts them, and the result does not depend on timing (the
 * partial products are added in a fixed order). */
MMTRAIN_API size_t mmtrain_gemm_workspace_bytes(int32_t layout, int32_t M, int32_t N);
MMTRAIN_API int mmtrain_gemm(int32_t dtype, int32_t layout, int32_t M, int32_t N, int32_t K,
                 const void *A, int32_t lda, const void *B, int32_t ldb, void *C, int32_t ldc,
                 const void *bias, const void *residual, uint32_t flags,
                 void *workspace, size_t workspace_bytes, void *hip_stream);

/* Bytes of workspace for the two attention operators below. */
MMTRAIN_API size_t mmtrain_attn_workspace_bytes(int32_t total_tokens, int32_t n_segments, int32_t n_heads);

/* Segment-masked attention forward over packed qkv[T, (nh + 2 nkv) d] (q heads | k heads |
 * v heads per row; rotary embedding, if any, already applied).  Writes o[T, nh d] and
 * lse[nh, T] (fp32 natural-log-sum-exp of the scaled, masked scores). */
MMTRAIN_API int mmtrain_attn_fwd(const mmtrain_layer_desc *desc, const mmtrain_batch *batch, const void *qkv,
                     void *o, float *lse, void *workspace, size_t workspace_bytes, void *hip_stream);

/* Attention backward: from d_o[T, nh d] and the forward's qkv, o, lse writes
 * d_qkv[T, (nh + 2 nkv) d] (same column order as qkv). */
MMTRAIN_API int mmtrain_attn_bwd(const mmtrain_layer_desc *desc, const mmtrain_batch *batch, const void *qkv,
                     const void *o, const float *lse, const void *d_o, void *d_qkv,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/* mmtrain_attn_bwd for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same arguments, results and
 * kernels as mmtrain_attn_bwd without the workspace: the scratch (per-token segment tables and the per-head
 * row sums D that the dQ kernel hands to the dK/dV kernel) is a fixed array of MMTRAIN_NOALLOC_SCRATCH_BYTES
 * inside the library, one copy on every GPU the library runs on, held until the process ends.  The call
 * allocates nothing and frees nothing, on the device or through any library.
 *   Limits: total_tokens <= MMTRAIN_NOALLOC_MAX_TOKENS and total_tokens * n_heads <=
 *   MMTRAIN_NOALLOC_MAX_HEAD_TOKENS, else MMTRAIN_ERR_TOO_LARGE (checked on the host, nothing enqueued).
 *   All calls on one GPU share that GPU's array, which keeps the previous call's contents; no entry has to
 *   start at zero (every entry read was written by the same call).  Calls on one stream are ordered and safe;
 *   calls that overlap on one GPU (different streams, different threads) race on the array.
 *   The first call on a device looks the array's address up (a host-side query, no allocation). */
#define MMTRAIN_NOALLOC_MAX_TOKENS 16384
#define MMTRAIN_NOALLOC_MAX_HEAD_TOKENS (64 * 16384)
#define MMTRAIN_NOALLOC_SCRATCH_BYTES (16384 * 4 + 16384 * 8 + 64 * 16384 * 4 + 4 * 256)
MMTRAIN_API int mmtrain_attn_bwd_noalloc(const mmtrain_layer_desc *desc, const mmtrain_batch *batch, const void *qkv,
                                         const void *o, const float *lse, const void *d_o, void *d_qkv,
                                         void *hip_stream);

/* Intra-microbatch reordering (Algorithm 1, Section "Intra-microbatch Reordering"): greedy multiway
 * partitioning of n samples over m data-parallel groups.  The samples are sorted by size in descending
 * order (equal sizes keep their original order) and handed out one by one to the group whose load is
 * currently the smallest (the lowest index among equals, which is what the paper's worked example
 * 1 2 3 4 -> 1 3 2 4 requires); the groups are then concatenated.
 *   sizes        host, [n]: cost of each sample, finite and >= 0 (tokens, or a time from a cost model such
 *                as a * tokens + b * attention pairs fitted to this library's measured step time)
 *   order        host, [n], out: order[p] = index of the sample at position p of the reordered batch
 *   group_begin  host, [m + 1], out, may be NULL: group j holds positions group_begin[j] .. group_begin[j+1]-1
 *   group_load   host, [m], out, may be NULL: sum of the sizes in each group
 * Host memory only, no GPU call, no allocation retained.  Returns MMTRAIN_OK, or MMTRAIN_ERR_INVALID_ARG
 * (n < 0, m <= 0, NULL sizes / order with n > 0, a negative, infinite or NaN size); nothing is written then. */
MMTRAIN_API int mmtrain_intra_reorder(const double *sizes, int32_t n, int32_t m, int32_t *order,
                                      int32_t *group_begin, double *group_load);

/* Timeline of a one-forward-one-backward (1F1B) pipeline over l microbatches and p stages (Section
 * "Inter-microbatch Reordering": an operation starts when the previous operation of its stage and the operation that
 * produces its input have both ended).  Stage s runs min(p-1-s, l) warm-up forward passes, then forward / backward
 * pairs, then the remaining backward passes.
 *   fwd, bwd   host, [p][l] row-major: duration of microbatch j's forward / backward pass on stage s at [s*l + j],
 *              finite and >= 0 (for this library: measured layer times x layers per stage, as a function of the pack)
 *   order      host, [l], may be NULL (identity): order[q] = index of the microbatch run at position q; a permutation
 *   makespan   host, out, may be NULL: end of the last operation
 *   intervals  host, [l], out, may be NULL: the first stage's pipeline intervals as the section defines them:
 *              intervals[0] = wait between the end of the first forward pass and the arrival of the first gradient
 *              (filled by forward passes 2..p); intervals[i-1], i >= 2 = wait between the end of backward pass i-1
 *              and the arrival of gradient i (filled by forward pass i+p-1; the last p-1 have nothing to fill them)
 * Host memory only, no GPU call.  Returns MMTRAIN_OK or MMTRAIN_ERR_INVALID_ARG (p < 1, l < 0, NULL fwd / bwd with
 * l > 0, a negative, infinite or NaN duration, an order that is not a permutation); nothing is written then. */
MMTRAIN_API int mmtrain_pipeline_1f1b(const double *fwd, const double *bwd, int32_t p, int32_t l, const int32_t *order,
                                      double *makespan, double *intervals);

/* Inter-microbatch reordering (Algorithm 2, Section "Inter-microbatch Reordering") for the 1F1B schedule above: the
 * smallest microbatch first, the p-1 smallest of the rest last (ascending), and in between, interval by interval, the
 * microbatches whose first-stage forward time comes closest to the interval's size (p-1 of them for the first
 * interval, each aiming at its share of what is still open; one for every later interval).  The interval sizes come
 * from the timeline of the microbatches placed so far, advanced by O(p) operations per placement.  Ties go to the
 * lowest index; the loop runs until no microbatch is left (the listing's l-p iterations would hand out l+p-2
 * microbatches).
 *   fwd, bwd        as above
 *   sizes           host, [l], may be NULL: the size of each microbatch for "smallest" -- the section defines it as the
 *                   microbatch's computation time in the modality encoder and the generator (the modules whose time
 *                   depends on the data), finite and >= 0.  NULL: forward + backward time of the first and the last stage,
 *                   i.e. the encoder's and the generator's stage of a pipeline encoder | backbone stages | generator; a
 *                   caller whose encoder or generator spans several stages passes the sum over those stages.
 *   order           host, [l], out: order[q] = index of the microbatch to run at position q
 *   intervals_seen  host, [l], out, may be NULL: the interval size each loop iteration worked with
 *   n_intervals     host, out, may be NULL: number of loop iterations (entries written to intervals_seen)
 * Host memory only, no GPU call.  Returns MMTRAIN_OK or MMTRAIN_ERR_INVALID_ARG (as above; NULL order with l > 0; a
 * negative, infinite or NaN size). */
MMTRAIN_API int mmtrain_inter_reorder(const double *fwd, const double *bwd, int32_t p, int32_t l, const double *sizes,
                                      int32_t *order, double *intervals_seen, int32_t *n_intervals);

/* Optimizer step of mixed-precision training with sharded optimizer state (Section 3: ZeRO-1 and mixed
 * precision for the LLM backbone; Section 4.2's memory constraint counts the optimizer state of one shard
 * per GPU).  One AdamW step, all in one pass over the shard:
 *     g = grad * grad_scale;  m = beta1 m + (1-beta1) g;  v = beta2 v + (1-beta2) g^2
 *     master -= lr * ( (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps) + weight_decay * master )
 *     param_out = master rounded to param_dtype;  grad = 0 if zero_grad
 * (the published Adam update with decoupled weight decay).  `grad` is the fp32 main-gradient buffer that
 * mmtrain_layer_bwd fills with MMTRAIN_BWD_WGRAD_F32 | MMTRAIN_BWD_ACCUMULATE_WGRAD.
 *   n                 elements in the shard (any value; 0 is a no-op)
 *   master, grad, exp_avg, exp_avg_sq   device, fp32 [n], 16-byte aligned, updated in place
 *   param_out         device, [n] of param_dtype (MMTRAIN_BF16 or MMTRAIN_F32), 16-byte aligned, may be NULL
 * Arithmetic in fp32; 1 - beta and the two bias corrections are evaluated in double on the host.  Enqueues one kernel on
 * hip_stream, allocates nothing, does not synchronise.  MMTRAIN_ERR_INVALID_ARG for a bad description
 * (struct_size, lr < 0, beta outside [0,1), eps <= 0, weight_decay < 0, step < 1), NULL or misaligned buffers. */
typedef struct {
    uint32_t struct_size;      /* sizeof(mmtrain_adam_desc) */
    float lr, beta1, beta2, eps, weight_decay;
    float grad_scale;          /* 1 / (number of microbatches accumulated), or an unscaling factor */
    int32_t step;              /* t >= 1, the step being taken */
    int32_t zero_grad;         /* non-zero: clear grad for the next accumulation */
} mmtrain_adam_desc;
MMTRAIN_API int mmtrain_adam_step(const mmtrain_adam_desc *desc, int64_t n, float *master, float *grad, float *exp_avg,
                                  float *exp_avg_sq, void *param_out, int32_t param_dtype, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* MMTRAIN_H */
