// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_16x16x32_bf16), fp32 accumulation.
//
//   C[M,N] (+)= opA(A) . opB(B) (+ bias[N]) (+ residual[M,N])
//
// Tiling.  One 256-thread workgroup (4 wavefronts, one per SIMD) owns a 256x256 tile of C;
// each wavefront owns a 128x128 quadrant as 8x8 MFMA tiles of 16x16 (256 accumulator
// registers per lane).  K advances in steps of 64; the 32 KiB operand tiles (256 rows x 64 k) of
// successive steps go round a ring of five LDS slots, which is all of the CU's 160 KiB.
//
// Global -> LDS.  Every operand tile is copied 16 bytes per lane directly into LDS (buffer_load ... lds:
// no register staging, no LDS write instructions), in the operand's own memory order, so weight- and
// input-gradient GEMMs need no transposed copies in HBM and no transposes in registers:
//   * operands whose contraction index is contiguous in memory (A of NT/NN, B of NT) are kept as
//     tile[row][64 k] (128 bytes = eight 16-byte units per row).  Unit u of row r is stored at unit
//     position u ^ (r & 7).  A fragment read (lane l: row l & 15, unit 4 s + (l >> 4), 16 bytes) is served 16
//     lanes at a time, lanes 0-7 together with 24-31 and 8-15 with 16-23 (measured), at full rate if those fall
//     into 16 distinct 16-byte slots modulo 256 bytes: rows 0-7 of one unit and rows 8-15 of its neighbour do
//     with this swizzle (with (r ^ (r >> 3)) & 7, which suits 32-row fragments, they ran at half rate);
//   * operands whose contraction index is the row index in memory (B of NN, A and B of TN) are kept as
//     tile[64 k][256 rows] (512 bytes per k) and the fragments are formed by the transposing LDS read
//     ds_read_b64_tr_b16; 32-byte chunks are XOR-swizzled with k & 3 against bank conflicts.
// Out-of-range rows and k are zero-filled by the buffer descriptor's bounds check.
//
// Epilogue.  Accumulators go through a per-wavefront fp32 LDS staging area so that C,
// residual and bias are accessed as full 16-byte row-major vectors; bias / residual / previous
// C (accumulate) are added in fp32 before the single rounding to bf16.
//
// Workgroup -> tile map.  The kernel is persistent: one workgroup per compute unit walks over
// several tiles, so the output stores of one tile drain while the next tile is already being
// multiplied.  Workgroups are dispatched round-robin over the 8 XCDs, each with its own L2; each
// XCD works on a contiguous run of the tile order, which goes in column-major groups of 8
// tile-rows so that concurrently resident tiles share A and B panels.
#include "kernels.h"
#include <atomic>
#include <utility>
#include <type_traits>

namespace mmt {

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int TILE_BYTES = BM * BK * 2;          // 32 KiB per operand tile
constexpr int N_SLOTS = 5;                       // ring of operand tiles: A0 B0 A1 B1 A2 | B2 A3 ...
constexpr int SMEM_BYTES = N_SLOTS * TILE_BYTES; // 160 KiB: all of the compute unit's LDS
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
    int c_f32;                 // C holds fp32 (weight gradients into fp32 main-gradient buffers)
    int tiles_m, tiles_n;
    // split K (fp32 output only): the K range is cut into `splits` chunks of k_chunk (a multiple of 64); chunk s of
    // every tile is a work item of its own and writes the partial product to C + s * split_stride (fp32 elements)
    int splits, k_chunk;
    long split_stride;
    // A launch covers tiles [tile_begin, tile_begin + tile_count) of the tile order.  With `compact` (fp32 output)
    // the partial product of chunk s of the launch's tile j is a dense 256 x 256 block at
    // C + (s * tile_count + j) * 65536 instead of a window of an M x N matrix.
    int tile_begin, tile_count, compact;
    unsigned long long *clock_probe;       // see GemmArgs
};

// Several products of one layout and epilogue in one launch (the weight gradients of a narrow layer, each with too few
// tiles to fill the chip): the work items of problem i are [first[i], first[i + 1]); first[i] for i >= n is the total.
constexpr int MAX_GROUP = 4;
struct GemmGroup {
    GemmP p[MAX_GROUP];
    int first[MAX_GROUP + 1];
    int n;
};
// what the kernel needs from its argument, for one product or a group
__device__ __forceinline__ const GemmP &first_problem(const GemmP &a) { return a; }
__device__ __forceinline__ const GemmP &first_problem(const GemmGroup &a) { return a.p[0]; }
__device__ __forceinline__ int work_items(const GemmP &a, bool split) { return a.tile_count * (split ? a.splits : 1); }
__device__ __forceinline__ int work_items(const GemmGroup &a, bool) { return a.first[MAX_GROUP]; }
// work item `logical` of the launch -> its problem and its index among that problem's items
__device__ __forceinline__ GemmP pick(const GemmP &a, int logical, int &local) { local = logical; return a; }
__device__ __forceinline__ GemmP pick(const GemmGroup &a, int logical, int &local) {
    GemmP p = a.p[0];
    local = logical;
    if (logical >= a.first[1]) { p = a.p[1]; local = logical - a.first[1]; }
    if (logical >= a.first[2]) { p = a.p[2]; local = logical - a.first[2]; }
    if (logical >= a.first[3]) { p = a.p[3]; local = logical - a.first[3]; }
    return p;
}

// position t of the tile order -> tile coordinates: column-major inside groups of GROUP_M tile-rows
__device__ __forceinline__ void tile_coords(int t, int tiles_m, int tiles_n, int &tm, int &tn) {
    const int width = GROUP_M * tiles_n;
    const int group = t / width, first_m = group * GROUP_M;
    const int gsize = min(tiles_m - first_m, GROUP_M);
    tm = first_m + (t % width) % gsize;
    tn = (t % width) / gsize;
}

__device__ __forceinline__ int swz(int row) { return row & 7; }

// Global memory is read through raw buffer descriptors: an access whose byte offset lies at or beyond
// the descriptor's size returns zero, which is how out-of-range rows and the K tail are zero-filled
// without branches.
constexpr uint32_t OOB = 0xfffffff0u;
typedef __attribute__((ext_vector_type(4))) uint32_t rawx4;

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void *p, size_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(p), 0, (int)(uint32_t)bytes, 0x00020000);
}
// the descriptor make_rsrc builds, as four scalar words
__device__ __forceinline__ rawx4 raw_rsrc(const void *p, size_t bytes) {
    const uint64_t a = (uint64_t)p;
    rawx4 r;
    r[0] = __builtin_amdgcn_readfirstlane((uint32_t)a);
    r[1] = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32) & 0xffffu);
    r[2] = __builtin_amdgcn_readfirstlane((uint32_t)bytes);
    r[3] = 0x00020000u;
    return r;
}
__device__ __forceinline__ uint4 buf_load(__amdgpu_buffer_rsrc_t r, uint32_t off) {
    const rawx4 v = __builtin_amdgcn_raw_buffer_load_b128(r, (int)off, 0, 0);
    return make_uint4(v[0], v[1], v[2], v[3]);
}

// K-contiguous operand: X[rows, K] row-major, copied global -> LDS without passing through registers
// (buffer_load ... lds).  One such instruction writes lane l's 16 bytes to LDS base + 16 l, i.e. one
// instruction fills 8 consecutive tile rows (1 KiB); the swizzled layout is obtained by choosing which
// 16-byte unit of the row each lane fetches: lane l of the slab starting at row r0 (a multiple of 8) fetches unit
// (l & 7) ^ swz(r0 + (l >> 3)) = (l & 7) ^ (l >> 3).  Wavefront w copies rows 32 i + 8 w .. + 7 for i = 0..7.
typedef __attribute__((address_space(3))) void lds_void;
struct LoaderKC {
    static constexpr int ITEM_LDS = 32 * 128;      // LDS bytes between consecutive items
    __amdgpu_buffer_rsrc_t rs;
    rawx4 rsv;                    // the same descriptor as four words, for the copies written as assembly
    uint32_t vo8[8];              // fast path: this lane's byte offset for item i, without k0
    __device__ __forceinline__ uint32_t step_soff(int k0) const { return (uint32_t)k0 * 2u; }
    uint32_t off0, row_step;      // byte offset of this lane's row at i = 0 (without the unit); bytes per 32 rows
    uint32_t vo_e, vo_o;          // fast path: this lane's byte offset for even / odd i, without k0 and i * row_step
    int kc0, K, slab0;            // unit column (elements) this lane fetches; first slab's LDS offset
    bool full;                    // all 256 rows of the tile exist
    __device__ __forceinline__ void init(const bf16_t *X, int ld, int row0, int nrows, int K_) {
        rs = make_rsrc(X, ((size_t)(nrows - 1) * ld + K_) * 2);
        const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
        K = K_;
        kc0 = (((lane & 7) ^ (lane >> 3)) & 7) * 8;
        off0 = (uint32_t)((size_t)(row0 + w * 8 + (lane >> 3)) * ld * 2);
        row_step = (uint32_t)ld * 64u;
        vo_e = off0 + (uint32_t)kc0 * 2u;
        vo_o = vo_e;
        full = row0 + BM <= nrows;
        slab0 = __builtin_amdgcn_readfirstlane(w * 8 * 128);
        // one register per item, kept there (recomputed inside the K loop they would cost a vector add per copy)
#pragma unroll
        for (int i = 0; i < 8; ++i) { vo8[i] = ((i & 1) ? vo_o : vo_e) + (uint32_t)i * row_step; asm volatile("" : "+v"(vo8[i])); }
        rsv = raw_rsrc(X, ((size_t)(nrows - 1) * ld + K_) * 2);
    }
    // item i of 8 of the tile at k0: rows 32 i + 8 w .. + 7 -> LDS.  FAST: the caller guarantees that the
    // tile lies inside the matrix (all rows, k0 + 64 <= K); then the per-lane offset is a constant and the
    // rest of the address is a scalar, so no vector instruction precedes the copy (a copy that has to wait
    // for the vector ALU to deliver its address holds up the MFMAs queued behind it).
    template <bool FAST>
    __device__ __forceinline__ void copy_one(uint8_t *tile, int k0, int i) const {
        lds_void *dst = (lds_void *)(tile + slab0 + i * 32 * 128);
        if (FAST) {
            const int so = __builtin_amdgcn_readfirstlane(k0 * 2 + i * (int)row_step);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, dst, 16, (int)((i & 1) ? vo_o : vo_e), so, 0, 0);
        } else {
            const int kc = kc0;
            const uint32_t off = k0 + kc < K ? off0 + i * row_step + (uint32_t)(k0 + kc) * 2u : OOB;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, dst, 16, (int)off, 0, 0, 0);
        }
    }
    __device__ __forceinline__ void copy_items(uint8_t *tile, int k0, int lo, int hi) const {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (i >= lo && i < hi) copy_one<false>(tile, k0, i);
    }
};

// K-strided operand: X[K, rows] row-major.  It is copied global -> LDS in its memory order, tile[k][row]
// with 512 bytes per k, by the same direct copies (one instruction = 2 k-rows), and the MFMA fragments
// are formed by the transposing LDS read (ds_read_b64_tr_b16): 16 lanes read a 4(k) x 16(row) block, 8
// bytes per lane, and lane j of the 16 receives the 4 k-values of row j.  Two such reads give a lane its
// 8 consecutive k.  The 32-byte chunk c of k-row k is stored at chunk position c ^ (k & 3), so that the 4
// k-rows of one block fall into different banks; the copy chooses which chunk each lane fetches.
// Wavefront w copies k-rows 16 w + 2 i, + 1 for i = 0..7.
typedef __attribute__((ext_vector_type(4))) short shortx4;
typedef __attribute__((ext_vector_type(8))) short shortx8;
typedef __attribute__((address_space(3))) shortx4 lds_shortx4;
struct LoaderKS {
    static constexpr int ITEM_LDS = 1024;
    __amdgpu_buffer_rsrc_t rs;
    rawx4 rsv;
    uint32_t vo8[8];
    __device__ __forceinline__ uint32_t step_soff(int k0) const { return (uint32_t)k0 * k_step; }
    uint32_t off_e, off_o, k_step;   // byte offset of this lane's 16 bytes for even / odd i (k0 = 0, i = 0 or 1); bytes per k
    int slab0;
    bool full;                       // all 256 rows of the tile exist
    __device__ __forceinline__ void init(const bf16_t *X, int ld, int row0, int nrows, int K_) {
        rs = make_rsrc(X, ((size_t)(K_ - 1) * ld + nrows) * 2);
        const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
        const int pos = lane & 31, kh = lane >> 5;            // 16-byte position in the k-row; which of the 2 k-rows
        const int n_e = (((pos >> 1) ^ kh) << 4) + (pos & 1) * 8;          // (k & 3) = kh for even i
        const int n_o = (((pos >> 1) ^ (2 + kh)) << 4) + (pos & 1) * 8;    //          2 + kh for odd i
        k_step = (uint32_t)ld * 2u;
        off_e = row0 + n_e < nrows ? (uint32_t)(((size_t)(w * 16 + kh) * ld + row0 + n_e) * 2) : OOB;
        off_o = row0 + n_o < nrows ? (uint32_t)(((size_t)(w * 16 + 2 + kh) * ld + row0 + n_o) * 2) : OOB;
        full = row0 + BM <= nrows;
        slab0 = __builtin_amdgcn_readfirstlane(w * 8 * 1024);
#pragma unroll
        for (int i = 0; i < 8; ++i) { vo8[i] = ((i & 1) ? off_o : off_e) + (uint32_t)(2 * (i & ~1)) * k_step; asm volatile("" : "+v"(vo8[i])); }
        rsv = raw_rsrc(X, ((size_t)(K_ - 1) * ld + nrows) * 2);
    }
    // FAST: as for the K-contiguous loader (all rows exist, k0 + 64 <= K).
    template <bool FAST>
    __device__ __forceinline__ void copy_one(uint8_t *tile, int k0, int i) const {
        const uint32_t base = (i & 1) ? off_o : off_e;
        lds_void *dst = (lds_void *)(tile + slab0 + i * 1024);
        if (FAST) {
            const int so = __builtin_amdgcn_readfirstlane((k0 + 2 * (i & ~1)) * (int)k_step);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, dst, 16, (int)base, so, 0, 0);
        } else {
            const uint32_t off = base == OOB ? OOB : base + (uint32_t)(k0 + 2 * (i & ~1)) * k_step;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, dst, 16, (int)off, 0, 0, 0);
        }
    }
    __device__ __forceinline__ void copy_items(uint8_t *tile, int k0, int lo, int hi) const {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (i >= lo && i < hi) copy_one<false>(tile, k0, i);
    }
};

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding
// global store to be acknowledged (its release fence), which would expose the latency of the output
// stores at each barrier; here only LDS operations (lgkmcnt) are waited for.  Direct-to-LDS copies are
// tracked by vmcnt and waited for separately where a stage is handed over.
__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}
// Orders this wavefront's own LDS writes before its later LDS reads (other lanes' data, same wavefront).
__device__ __forceinline__ void lds_wave_sync() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// Fragment reads issued as assembly.  The compiler makes every LDS read that it cannot prove independent
// of an older direct-to-LDS copy wait for that copy (vmcnt), which it does for the transposing read; written
// as assembly the read carries no such wait.  The price is that the compiler does not know when the data
// arrive: every use is preceded by an explicit s_waitcnt lgkmcnt (wait_frags below), which names the fragment
// registers as operands so that the MFMAs that consume them cannot be moved in front of it.
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_tr(uint32_t addr) {
    shortx4 lo, hi;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(addr), "n"(OFF));
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(addr), "n"(OFF + 4 * 512));
    const shortx8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return *reinterpret_cast<const bf16x8 *>(&v);
}
template <int OFF>
__device__ __forceinline__ bf16x8 lds_read_b128(uint32_t addr) {
    bf16x8 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
    return v;
}
// The 16 fragments of a 32-deep k-slice (8 of A, 8 of B, 16 rows each) are read in the order
// A0 B0 .. B7 A1 .. A7, one per MFMA group, one slice ahead.  MFMA group g of a slice (row block g >> 1
// of A against four of the B fragments) needs the fragments up to position need(g); LDS reads return in
// order, so the group may proceed once at most this many LDS instructions are outstanding: the previous
// slice's reads behind that position plus this slice's reads issued so far (groups 0..g-1: a group's own
// read follows its first MFMA).  The counter holds 15 at most.
constexpr int frag_is_a(int f) { return f == 0 || f >= 9; }
constexpr int frag_index(int f) { return f == 0 ? 0 : f <= 8 ? f - 1 : f - 8; }
template <bool A_KC, bool B_KC>
constexpr int lgkm_allowed(int g) {
    const int ca = A_KC ? 1 : 2, cb = B_KC ? 1 : 2;
    const int need = g == 0 ? 4 : g == 1 ? 8 : 8 + (g >> 1);
    int n = 0;
    for (int f = need + 1; f < 16; ++f) n += frag_is_a(f) ? ca : cb;
    for (int f = 0; f < g; ++f) n += frag_is_a(f) ? ca : cb;
    return n < 15 ? n : 15;
}
template <int N>
__device__ __forceinline__ void wait_frags(bf16x8 &a, bf16x8 &b, bf16x8 &c, bf16x8 &d, bf16x8 &e) {
    asm volatile("s_waitcnt lgkmcnt(%5)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d), "+v"(e) : "n"(N));
}
template <int N>
__device__ __forceinline__ void wait_frags(bf16x8 &a, bf16x8 &b, bf16x8 &c, bf16x8 &d) {
    asm volatile("s_waitcnt lgkmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N));
}
template <int N>
__device__ __forceinline__ void wait_frags(bf16x8 &a) {
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(a) : "n"(N));
}
template <int... I, class F>
__device__ __forceinline__ void static_for(std::integer_sequence<int, I...>, F &&f) {
    (f(std::integral_constant<int, I>{}), ...);
}

// One MFMA with the copy of one item of an operand tile behind it, as one statement: M0 (the LDS destination) is written in
// front of the MFMA, which also is the wait state the copy needs after that write, and the copy's scalar offset is the same for
// all items of a step (the builtin form costs a scalar add for the offset, one for M0 and a no-op per copy).
template <int MOFF>
__device__ __forceinline__ void mfma_copy(f32x4 &acc, const bf16x8 &b, const bf16x8 &a, uint32_t mbase, uint32_t vo, const rawx4 &rsv,
                                          uint32_t so) {
    asm volatile("s_add_u32 m0, %[mb], %[moff]\n\tv_mfma_f32_16x16x32_bf16 %[acc], %[b], %[a], %[acc]\n\t"
                 "buffer_load_dwordx4 %[vo], %[rs], %[so] offen lds"
                 : [acc] "+a"(acc) : [b] "v"(b), [a] "v"(a), [mb] "s"(mbase), [moff] "n"(MOFF), [vo] "v"(vo), [rs] "s"(rsv), [so] "s"(so)
                 : "memory", "m0", "scc");
}

template <bool KC> struct LoaderSel { typedef LoaderKC type; };
template <> struct LoaderSel<false> { typedef LoaderKS type; };

template <bool A_KC, bool B_KC, bool HAS_ADD, bool OUT_F32, typename ARG = GemmP>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1)))
void gemm_mfma_kernel(const ARG arg) {
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const unsigned long long *const probe_ = first_problem(arg).clock_probe;
    unsigned long long *const clock_probe = const_cast<unsigned long long *>(probe_);

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    if (clock_probe && blockIdx.x == 0 && threadIdx.x == 0) {
        clock_probe[0] = (unsigned long long)clock64();
        clock_probe[1] = (unsigned long long)wall_clock64();
    }

    // ---- persistent workgroup -> tiles.  Workgroup b runs on XCD b % 8 (round-robin dispatch); XCD x
    // owns a contiguous run of the tile order, and its workgroups stride through that run together.
    const int ntiles = work_items(arg, OUT_F32);                  // work items: (K chunk, tile), chunk-major
    const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
    const int per = ntiles >> 3, rem = ntiles & 7;
    const int run_begin = xcd < rem ? xcd * (per + 1) : rem * (per + 1) + (xcd - rem) * per;
    const int run_end = run_begin + per + (xcd < rem ? 1 : 0);
    const int wg_per_xcd = (gridDim.x - xcd + 7) >> 3;

    // fragment addressing (v_mfma_f32_16x16x32_bf16: lane l holds row l & 15, k = 8 (l >> 4) .. + 7 of a
    // 16-row, 32-deep fragment).  K-contiguous tile: row block i, slice s -> row 16 i + (l & 15), unit
    // 4 s + (l >> 4); the swizzle of that row is that of row l & 15, so two offsets per operand (one per slice)
    // cover all blocks, the block itself being an immediate offset of the read.  K-strided tile: the 16 lanes with
    // the same l >> 4 form rows 0..15 of the block at k = 8 (l >> 4) ..; lane j of them supplies the address
    // of k-row (j >> 2), rows 4 (j & 3) .. + 3, for each of the two transposing reads.
    const int frow = lane & 15, fq = lane >> 4;
    int a_rd[4][2], b_rd[4][2];
#pragma unroll
    for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int sl = 0; sl < 2; ++sl) {
            if (A_KC) a_rd[c][sl] = (wm * 128 + frow) * 128 + (((sl * 4 + fq) ^ swz(frow)) << 4);
            else a_rd[c][sl] = (sl * 32 + 8 * fq + (frow >> 2)) * 512 + (frow & 3) * 8 + ((wm * 8 + c) ^ (frow >> 2)) * 32;
            if (B_KC) b_rd[c][sl] = (wn * 128 + frow) * 128 + (((sl * 4 + fq) ^ swz(frow)) << 4);
            else b_rd[c][sl] = (sl * 32 + 8 * fq + (frow >> 2)) * 512 + (frow & 3) * 8 + ((wn * 8 + c) ^ (frow >> 2)) * 32;
        }

    for (int logical = run_begin + q; logical < run_end; logical += wg_per_xcd) {
    int tm, tn, item;
    const GemmP p = pick(arg, logical, item);                  // (a group: the problem this work item belongs to)
    const int chunk = OUT_F32 ? item / p.tile_count : 0;
    const int tl = item - chunk * p.tile_count;                // tile within this launch
    tile_coords(p.tile_begin + tl, p.tiles_m, p.tiles_n, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    // this work item's K range (only the fp32-output kernels are ever split)
    const int k_begin = OUT_F32 ? chunk * p.k_chunk : 0;
    const int Kc = OUT_F32 ? min(p.k_chunk, p.K - k_begin) : p.K;

    typename LoaderSel<A_KC>::type la;
    typename LoaderSel<B_KC>::type lb;
    la.init(p.A + (size_t)k_begin * (A_KC ? 1 : p.lda), p.lda, m0, p.M, Kc);
    lb.init(p.B + (size_t)k_begin * (B_KC ? 1 : p.ldb), p.ldb, n0, p.N, Kc);

    f32x4 acc[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

    bf16x8 fa[2][8], fb[2][8];
    // Kernels with a K-strided operand read all their fragments as assembly (see lds_read_tr) and wait for
    // them explicitly; the all-K-contiguous kernel leaves reads and waits to the compiler.
    constexpr bool ASM_READS = !(A_KC && B_KC);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(lds_void *)smem;
    // fragment f of 16 of slice SL (0, 1) of the tiles at LDS offsets ta, tb, into fragment buffer buf
    auto read_frag = [&](auto SL, auto F, int ta, int tb, int buf) {
        constexpr int sl = decltype(SL)::value, f = decltype(F)::value;
        constexpr bool is_a = frag_is_a(f);
        constexpr int i = frag_index(f);
        // K-contiguous: all blocks share the swizzle term; K-strided: one offset per pair (wave half, block)
        constexpr int kc_imm = i * 16 * 128, c_kc = i & 3;
        constexpr int ks_imm = (i >> 2) * 4 * 32, c_ks = i & 3;     // chunk (wm * 8 + i): bits 0..1 in the offset, bit 2 immediate
        if (is_a) {
            if (A_KC) {
                if (!ASM_READS) fa[buf][i] = *reinterpret_cast<const bf16x8 *>(smem + ta + a_rd[c_kc][sl] + kc_imm);
                else fa[buf][i] = lds_read_b128<kc_imm>(lds0 + ta + a_rd[c_kc][sl]);
            } else fa[buf][i] = lds_read_tr<ks_imm>(lds0 + ta + a_rd[c_ks][sl]);
        } else {
            if (B_KC) {
                if (!ASM_READS) fb[buf][i] = *reinterpret_cast<const bf16x8 *>(smem + tb + b_rd[c_kc][sl] + kc_imm);
                else fb[buf][i] = lds_read_b128<kc_imm>(lds0 + tb + b_rd[c_kc][sl]);
            } else fb[buf][i] = lds_read_tr<ks_imm>(lds0 + tb + b_rd[c_ks][sl]);
        }
    };
    // before MFMA group g (0..15) of a slice held in fragment buffer `buf`
    auto wait_group = [&](auto G, int buf) {
        constexpr int g = decltype(G)::value;
        constexpr int n = lgkm_allowed<A_KC, B_KC>(g);
        if (!ASM_READS) return;
        if (g == 0) wait_frags<n>(fa[buf][0], fb[buf][0], fb[buf][1], fb[buf][2], fb[buf][3]);
        else if (g == 1) wait_frags<n>(fb[buf][4], fb[buf][5], fb[buf][6], fb[buf][7]);
        else if (!(g & 1)) wait_frags<n>(fa[buf][g >> 1]);
    };
    // MFMA group g of 16 of a k-slice: row block i = g >> 1 of A against B blocks 4 (g & 1) .. + 3.
    // Operands are swapped: the accumulator tile is held transposed (lane = m, registers run over n),
    // so that each lane owns 4 consecutive n of one row for the epilogue.  The instruction is written out
    // with the accumulator tied to itself in the accumulation registers: left to the register allocator,
    // the 64 four-register accumulators are shuffled between registers in every iteration.  An
    // accumulator is touched again only 64 MFMAs later, and the code after the K loop starts with waits
    // and a barrier, so none of the software-managed MFMA hazards can occur.
    auto mfma = [&](int buf, int g, int t) {
        const int i = g >> 1, j = 4 * (g & 1);
        asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j + t]) : "v"(fb[buf][j + t]), "v"(fa[buf][i]));
    };

    // Software pipeline, one barrier per 64-deep K step.  The operand tiles A0 B0 A1 B1 A2 B2 ... go round
    // a ring of five 32 KiB slots.  Step kt multiplies K tile kt in two 32-deep k-slices of 16 MFMA groups
    // (4 MFMAs = 64 cycles each); every group also reads one fragment of the following slice, so after the
    // first slice every wavefront has read all of A(kt) and B(kt): past the barrier in the middle of the
    // step their two slots are handed to B(kt+2) and A(kt+3), and the second slice's groups read the first
    // slice of tile kt+1.  Between two barriers a wavefront issues the 8 copies of one B tile and then the 8
    // copies of one A tile, one in every second MFMA group: the compute unit's address path takes about 20
    // cycles per 1 KiB copy, and four wavefronts issuing one in every group would back it up and stall
    // the MFMAs behind it.  At the barrier of step kt the tiles A(kt+1) (copied during the previous step)
    // and B(kt+1) (copied in the first half of this interval) must have landed; the 8 youngest copies (of
    // A(kt+2)) may still be in flight (vmcnt(8): memory operations retire in issue order).  A copy thus
    // has between one and three slices to land, against about half a slice of L2 latency.
    const int nk = (Kc + BK - 1) / BK;
    typedef std::integral_constant<int, 0> S0;
    typedef std::integral_constant<int, 1> S1;
    typedef std::make_integer_sequence<int, 16> Groups16;
    la.copy_items(smem + 0 * TILE_BYTES, 0, 0, 8);
    lb.copy_items(smem + 1 * TILE_BYTES, 0, 0, 8);
    la.copy_items(smem + 2 * TILE_BYTES, BK, 0, 8);
    lb.copy_items(smem + 3 * TILE_BYTES, BK, 0, 8);
    asm volatile("s_waitcnt vmcnt(16)" ::: "memory");         // A0 and B0 have landed
    lds_barrier();
    static_for(Groups16{}, [&](auto G) { read_frag(S0{}, G, 0, TILE_BYTES, 0); });

    // LDS offsets of the slots that hold tiles 2kt .. 2kt+4 of the ring (A(kt), B(kt), A(kt+1), B(kt+1), A(kt+2))
    int o0 = 0, o1 = TILE_BYTES, o2 = 2 * TILE_BYTES, o3 = 3 * TILE_BYTES, o4 = 4 * TILE_BYTES;
    const bool full_tiles = la.full && lb.full;
    auto step = [&](auto FAST_, int kt) {
        constexpr bool FAST = decltype(FAST_)::value;
        const int k2 = (kt + 2) * BK;
        typedef std::remove_reference_t<decltype(la)> LA;
        typedef std::remove_reference_t<decltype(lb)> LB;
        // fast path: scalar offsets and LDS destinations of this step's copies
        const uint32_t so_a = __builtin_amdgcn_readfirstlane(la.step_soff(k2)), so_b = __builtin_amdgcn_readfirstlane(lb.step_soff(k2));
        const uint32_t mb_a = __builtin_amdgcn_readfirstlane(lds0 + o4 + la.slab0), mb_b = __builtin_amdgcn_readfirstlane(lds0 + o0 + lb.slab0);
        // first slice: fragments of the second slice; A(kt+2) into the slot B(kt-1) had
        static_for(Groups16{}, [&](auto G) {
            constexpr int g = decltype(G)::value;
            wait_group(G, 0);
            mfma(0, g, 0);
            __builtin_amdgcn_sched_barrier(0);
            read_frag(S1{}, G, o0, o1, 1);
            __builtin_amdgcn_sched_barrier(0);
            if (FAST && !(g & 1))
                mfma_copy<(g >> 1) * LA::ITEM_LDS>(acc[g >> 1][4 * (g & 1) + 1], fb[0][4 * (g & 1) + 1], fa[0][g >> 1], mb_a, la.vo8[g >> 1], la.rsv, so_a);
            else mfma(0, g, 1);
            __builtin_amdgcn_sched_barrier(0);
            if (!FAST && !(g & 1)) la.template copy_one<false>(smem + o4, k2, g >> 1);
            __builtin_amdgcn_sched_barrier(0);
            mfma(0, g, 2);
            mfma(0, g, 3);
            __builtin_amdgcn_sched_barrier(0);
        });
        asm volatile("s_waitcnt vmcnt(8)" ::: "memory");       // A(kt+1) and B(kt+1) have landed
        lds_barrier();                                         // and nobody reads A(kt), B(kt) any more
        // second slice: fragments of the first slice of tile kt+1; B(kt+2) into the slot A(kt) had.
        // The barrier has waited for every LDS read, so this slice's MFMAs need no wait of their own.
        static_for(Groups16{}, [&](auto G) {
            constexpr int g = decltype(G)::value;
            if (ASM_READS && g == 0)       // ties the MFMAs below to this side of the barrier
                asm volatile("" : "+v"(fa[1][0]), "+v"(fa[1][1]), "+v"(fa[1][2]), "+v"(fa[1][3]),
                                  "+v"(fa[1][4]), "+v"(fa[1][5]), "+v"(fa[1][6]), "+v"(fa[1][7]),
                                  "+v"(fb[1][0]), "+v"(fb[1][1]), "+v"(fb[1][2]), "+v"(fb[1][3]),
                                  "+v"(fb[1][4]), "+v"(fb[1][5]), "+v"(fb[1][6]), "+v"(fb[1][7]));
            mfma(1, g, 0);
            __builtin_amdgcn_sched_barrier(0);
            read_frag(S0{}, G, o2, o3, 0);
            __builtin_amdgcn_sched_barrier(0);
            if (FAST && !(g & 1))
                mfma_copy<(g >> 1) * LB::ITEM_LDS>(acc[g >> 1][4 * (g & 1) + 1], fb[1][4 * (g & 1) + 1], fa[1][g >> 1], mb_b, lb.vo8[g >> 1], lb.rsv, so_b);
            else mfma(1, g, 1);
            __builtin_amdgcn_sched_barrier(0);
            if (!FAST && !(g & 1)) lb.template copy_one<false>(smem + o0, k2, g >> 1);
            __builtin_amdgcn_sched_barrier(0);
            mfma(1, g, 2);
            mfma(1, g, 3);
            __builtin_amdgcn_sched_barrier(0);
        });
        { const int t0 = o0, t1 = o1; o0 = o2; o1 = o3; o2 = o4; o3 = t0; o4 = t1; }
    };
    // copies of a step reach up to K tile kt+2: the unchecked form needs that tile inside the matrix
    const int nk_fast = full_tiles ? max(Kc / BK - 2, 0) : 0;
    for (int kt = 0; kt < nk_fast; ++kt) step(std::true_type{}, kt);
    for (int kt = nk_fast; kt < nk; ++kt) step(std::false_type{}, kt);
    asm volatile("s_nop 15\n\ts_waitcnt vmcnt(0)" ::: "memory");   // the last MFMAs have written their accumulators;
                                                                  // copies past the end of K (zero-filled) are done
    if (ASM_READS) {
        // the last slice's reads (never used) still target these registers: keep them reserved until they land
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(fa[0][0]), "+v"(fa[0][1]), "+v"(fa[0][2]), "+v"(fa[0][3]),
                       "+v"(fa[0][4]), "+v"(fa[0][5]), "+v"(fa[0][6]), "+v"(fa[0][7]),
                       "+v"(fb[0][0]), "+v"(fb[0][1]), "+v"(fb[0][2]), "+v"(fb[0][3]),
                       "+v"(fb[0][4]), "+v"(fb[0][5]), "+v"(fb[0][6]), "+v"(fb[0][7]));
    }
    lds_barrier();

    // ---- epilogue: 32 rows x 128 columns at a time through this wavefront's own staging area; the output
    // stores are left in flight (nothing below waits for them) and drain under the next tile's K loop
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
    // Everything that is added to the product (residual, previous C) is fetched before the first output
    // store is issued: memory operations retire in order, so a load issued after a store would have to
    // wait for that store to be acknowledged.
    const bf16_t *addend = p.residual ? p.residual : p.C;      // HAS_ADD: residual and / or accumulate
    uint4 add[HAS_ADD ? 4 : 1][8];
    if (HAS_ADD) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int pass = 0; pass < 8; ++pass) {
                const int gm = m0 + wm * 128 + i * 32 + pass * 4 + er;
                add[i][pass] = make_uint4(0, 0, 0, 0);
                if (gm < p.M && nok) add[i][pass] = *reinterpret_cast<const uint4 *>(addend + (size_t)gm * p.ldc + gn);
            }
    }
    const bool both = HAS_ADD && p.residual && p.accumulate;   // rare: the second addend is read in the store loop
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // accumulator tile (2 i + ii, j), register e  <->  m = 16 (2 i + ii) + (lane & 15),  n = 16 j + 4 (lane >> 4) + e
#pragma unroll
        for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const f32x4 t = acc[2 * i + ii][j];
                *reinterpret_cast<float4 *>(stg + (ii * 16 + frow) * EPI_PITCH + j * 16 + fq * 4) = make_float4(t[0], t[1], t[2], t[3]);
            }
        lds_wave_sync();
#pragma unroll
        for (int pass = 0; pass < 8; ++pass) {
            const int r = pass * 4 + er;
            const int gm = m0 + wm * 128 + i * 32 + r;
            if (gm < p.M && nok) {
                const float4 v0 = *reinterpret_cast<const float4 *>(stg + r * EPI_PITCH + ec);
                const float4 v1 = *reinterpret_cast<const float4 *>(stg + r * EPI_PITCH + ec + 4);
                float v[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
                if (p.bias) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) v[e] += bv[e];
                }
                const size_t off = (size_t)gm * p.ldc + gn;
                if (HAS_ADD) {
                    const uint32_t w[4] = {add[i][pass].x, add[i][pass].y, add[i][pass].z, add[i][pass].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) { v[2 * e] += __uint_as_float(w[e] << 16); v[2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u); }
                }
                if (both) {
                    const uint4 raw = *reinterpret_cast<const uint4 *>(p.C + off);
                    const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) { v[2 * e] += __uint_as_float(w[e] << 16); v[2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u); }
                }
                if (OUT_F32) {
                    // fp32 output (never together with bias or residual): previous contents are read here
                    float *cf = reinterpret_cast<float *>(p.C) +
                                (p.compact ? ((size_t)(chunk * p.tile_count + tl) << 16) + (size_t)(gm - m0) * BN + (gn - n0)
                                           : (size_t)chunk * p.split_stride + off);
                    if (p.accumulate) {
                        const float4 c0 = *reinterpret_cast<const float4 *>(cf), c1 = *reinterpret_cast<const float4 *>(cf + 4);
                        v[0] += c0.x; v[1] += c0.y; v[2] += c0.z; v[3] += c0.w;
                        v[4] += c1.x; v[5] += c1.y; v[6] += c1.z; v[7] += c1.w;
                    }
                    __builtin_nontemporal_store(f32x4{v[0], v[1], v[2], v[3]}, reinterpret_cast<f32x4 *>(cf));
                    __builtin_nontemporal_store(f32x4{v[4], v[5], v[6], v[7]}, reinterpret_cast<f32x4 *>(cf + 4));
                    continue;
                }
                uint4 o;
                o.x = pack_bf16x2(v[0], v[1]); o.y = pack_bf16x2(v[2], v[3]);
                o.z = pack_bf16x2(v[4], v[5]); o.w = pack_bf16x2(v[6], v[7]);
                // streaming store: the output is not read again by this kernel, so it should not displace
                // operand panels from the L2
                __builtin_nontemporal_store(*reinterpret_cast<const rawx4 *>(&o), reinterpret_cast<rawx4 *>(p.C + off));
            }
        }
        lds_wave_sync();
    }
    lds_barrier();      // staging area is free again: the next tile's first stage may overwrite it
    }   // tiles of this workgroup
    if (clock_probe && blockIdx.x == 0 && threadIdx.x == 0) {
        clock_probe[2] = (unsigned long long)clock64();
        clock_probe[3] = (unsigned long long)wall_clock64();
    }
}

// compute units of the current device, rounded down to whole XCD octets (one persistent workgroup each)
hipError_t compute_units(int &n) {
    static std::atomic<int> cached{0};
    int n_cu = cached.load(std::memory_order_relaxed);
    if (n_cu == 0) {
        int dev = 0, v = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        if (v <= 0) v = 256;
        v &= ~7;
        n_cu = v ? v : 8;
        cached.store(n_cu, std::memory_order_relaxed);
    }
    n = n_cu;
    return hipSuccess;
}

template <bool A_KC, bool B_KC, bool HAS_ADD, bool OUT_F32 = false>
hipError_t launch(const GemmP &p, hipStream_t st) {
    static std::atomic<bool> configured{false};     // set once; concurrent first calls repeat the same idempotent set-up
    auto kern = gemm_mfma_kernel<A_KC, B_KC, HAS_ADD, OUT_F32>;
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    // one persistent workgroup per compute unit (the tile needs the CU's whole LDS and register file)
    int n_cu = 0;
    hipError_t e = compute_units(n_cu);
    if (e != hipSuccess) return e;
    const int items = p.tile_count * (OUT_F32 ? p.splits : 1);
    if (items <= 0) return hipSuccess;
    kern<<<items < n_cu ? items : n_cu, 256, SMEM_BYTES, st>>>(p);
    return hipGetLastError();
}

template <bool HAS_ADD, bool OUT_F32>
hipError_t launch_group_tn(const GemmGroup &g, hipStream_t st) {
    static std::atomic<bool> configured{false};     // set once; concurrent first calls repeat the same idempotent set-up
    auto kern = gemm_mfma_kernel<false, false, HAS_ADD, OUT_F32, GemmGroup>;
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    int n_cu = 0;
    hipError_t e = compute_units(n_cu);
    if (e != hipSuccess) return e;
    const int items = g.first[MAX_GROUP];
    if (items <= 0) return hipSuccess;
    kern<<<items < n_cu ? items : n_cu, 256, SMEM_BYTES, st>>>(g);
    return hipGetLastError();
}

// C (+)= sum over the K chunks of the fp32 partial products; C is bf16 or fp32.  4 elements per thread.
template <typename TC>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *__restrict__ part, int splits, long stride, int M, int N,
                                                            TC *__restrict__ C, int ldc, int accumulate) {
    const long idx = ((long)blockIdx.x * 256 + threadIdx.x) * 4;
    if (idx >= (long)M * N) return;
    const int m = (int)(idx / N), n = (int)(idx % N);                 // N is a multiple of 8
    f32x4 v = *reinterpret_cast<const f32x4 *>(part + idx);
    for (int sp = 1; sp < splits; ++sp) v += *reinterpret_cast<const f32x4 *>(part + sp * stride + idx);
    TC *c = C + (long)m * ldc + n;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float r = v[e];
        if (accumulate) r += Elem<TC>::load(c + e);
        Elem<TC>::store(c + e, r);
    }
}

// The same for the dense 256 x 256 partial blocks of the tiles [tile_begin, tile_begin + tile_count) of the tile
// order: block (s * tile_count + j) belongs to chunk s of tile tile_begin + j.  64 workgroups per tile.
template <typename TC>
__global__ __launch_bounds__(256) void tail_reduce_kernel(const float *__restrict__ part, int splits, int tile_begin, int tile_count,
                                                          int tiles_m, int tiles_n, int M, int N, TC *__restrict__ C, int ldc,
                                                          int accumulate) {
    const int j = blockIdx.x >> 6;
    const int e0 = ((blockIdx.x & 63) * 256 + threadIdx.x) * 4;         // element of the block: row e0 / 256, column e0 % 256
    int tm, tn;
    tile_coords(tile_begin + j, tiles_m, tiles_n, tm, tn);
    const int m = tm * BM + (e0 >> 8), n = tn * BN + (e0 & 255);
    if (m >= M || n >= N) return;                                       // N is a multiple of 8: the 4 columns are in or out together
    f32x4 v = *reinterpret_cast<const f32x4 *>(part + ((size_t)j << 16) + e0);
    for (int sp = 1; sp < splits; ++sp) v += *reinterpret_cast<const f32x4 *>(part + ((size_t)(sp * tile_count + j) << 16) + e0);
    TC *c = C + (size_t)m * ldc + n;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float r = v[e];
        if (accumulate) r += Elem<TC>::load(c + e);
        Elem<TC>::store(c + e, r);
    }
}

GemmP params(const GemmArgs &g) {
    GemmP p;
    p.M = g.M; p.N = g.N; p.K = g.K;
    p.A = (const bf16_t *)g.A; p.lda = g.lda;
    p.B = (const bf16_t *)g.B; p.ldb = g.ldb;
    p.C = (bf16_t *)g.C; p.ldc = g.ldc;
    p.bias = (const bf16_t *)g.bias;
    p.residual = (const bf16_t *)g.residual;
    p.accumulate = g.accumulate ? 1 : 0;
    p.c_f32 = g.c_f32 ? 1 : 0;
    p.tiles_m = ceil_div(g.M, BM);
    p.tiles_n = ceil_div(g.N, BN);
    p.splits = 1; p.k_chunk = g.K; p.split_stride = 0;
    p.tile_begin = 0; p.tile_count = p.tiles_m * p.tiles_n; p.compact = 0;
    p.clock_probe = g.clock_probe;
    return p;
}

// all K chunks of the tiles p covers as fp32 partial products (p.C: scratch)
hipError_t launch_partials(int layout, const GemmP &p, hipStream_t st) {
    return layout == GEMM_TN ? launch<false, false, false, true>(p, st) : launch<true, false, false, true>(p, st);
}

}  // namespace

bool gemm_mfma_supported(const GemmArgs &g) {
    if (g.M <= 0 || g.N <= 0 || g.K <= 0) return false;
    if (g.c_f32 && (g.layout != GEMM_TN || g.bias || g.residual)) return false;   // fp32 output: weight gradients only
    if ((g.lda | g.ldb | g.ldc | g.N) & 7) return false;
    const bool a_kc = g.layout != GEMM_TN, b_kc = g.layout == GEMM_NT;
    if ((a_kc || b_kc) && (g.K & 7)) return false;
    if (!a_kc && (g.M & 7)) return false;
    // operands are addressed with 32-bit byte offsets, tile overhang included
    const size_t rows_a = a_kc ? g.M : g.K, rows_b = b_kc ? g.N : g.K;
    if ((rows_a + 256) * (size_t)g.lda * 2 >= 0xfff00000ull || (rows_b + 256) * (size_t)g.ldb * 2 >= 0xfff00000ull)
        return false;
    const uintptr_t bits = (uintptr_t)g.A | (uintptr_t)g.B | (uintptr_t)g.C | (uintptr_t)g.bias | (uintptr_t)g.residual;
    return (bits & 15) == 0;
}

// How many K chunks for a weight-gradient GEMM: enough to give every compute unit a work item when the
// output has few tiles (a ViT-sized layer: 16 to 64 tiles against 256 compute units, K = all tokens of the
// pack), chunks of at least 512, and the partial products must fit the scratch buffer.
int gemm_mfma_splits(const GemmArgs &g) {
    if (g.layout != GEMM_TN || !g.split_ws || g.bias || g.residual) return 1;
    const long tiles = (long)ceil_div(g.M, BM) * ceil_div(g.N, BN);
    if (tiles > 128) return 1;
    long s = 256 / tiles;
    s = s < g.K / 512 ? s : g.K / 512;
    const long fit = (long)(g.split_ws_bytes / ((size_t)g.M * g.N * 4));
    s = s < fit ? s : fit;
    s = s < 32 ? s : 32;
    return s >= 2 ? (int)s : 1;
}

// The last, partly filled round of a large GEMM.  With one workgroup per compute unit the tiles are worked off in
// rounds of n_cu; when the last round holds at most half that many tiles, each of them is cut along K into
// n_cu / tiles chunks so that the round takes a fraction of a full one.  Returns the number of chunks (1: do not
// split) and the number of tiles in that round.  Only for input- and weight-gradient GEMMs without bias or
// residual, with scratch for the partial products, and only for long K: a partly filled round is faster than a full
// one to begin with (fewer active compute units run at a higher clock), and the cut costs two extra launches.
// Measured on the 22016 x 4096 x 8192 weight gradient (96 tiles in the last round, 2 chunks): 1.137 -> 1.100 ms; the
// 8192 x 11008 x 4096 input gradient gains nothing, hence the bound on K.
int gemm_mfma_tail_splits(const GemmArgs &g, int n_cu, int &tail_tiles) {
    tail_tiles = 0;
    if (g.layout == GEMM_NT || !g.split_ws || g.bias || g.residual) return 1;
    const long tiles = (long)ceil_div(g.M, BM) * ceil_div(g.N, BN);
    const long rem = tiles % n_cu;
    if (tiles < n_cu || rem == 0 || rem > n_cu / 2) return 1;
    long s = n_cu / rem;
    s = s < g.K / 512 ? s : g.K / 512;
    s = s < 16 ? s : 16;
    const long fit = (long)(g.split_ws_bytes / ((size_t)rem * BM * BN * 4));
    s = s < fit ? s : fit;
    if (s < 2 || (long)g.K * (s - 1) / s < 4096) return 1;
    tail_tiles = (int)rem;
    return (int)s;
}

// Weight-gradient products whose outputs have few tiles (at most 128: a narrow layer), run together: every tile of every
// product is one work item with the whole contraction, so nothing is cut along K, nothing goes through scratch and one
// launch fills the chip that each product alone would leave mostly idle.
bool gemm_mfma_few_tiles(const GemmArgs &g) {
    return g.layout == GEMM_TN && !g.bias && !g.residual && gemm_mfma_supported(g) &&
           (long)ceil_div(g.M, BM) * ceil_div(g.N, BN) <= 128;
}

hipError_t gemm_mfma_group(const GemmArgs *gs, int n, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    if (n > MAX_GROUP) return hipErrorInvalidValue;
    GemmGroup grp = {};
    int total = 0;
    for (int i = 0; i < n; ++i) {
        if (!gemm_mfma_few_tiles(gs[i]) || gs[i].accumulate != gs[0].accumulate || gs[i].c_f32 != gs[0].c_f32)
            return hipErrorInvalidValue;
        grp.p[i] = params(gs[i]);
        grp.first[i] = total;
        total += grp.p[i].tile_count;
    }
    for (int i = n; i <= MAX_GROUP; ++i) grp.first[i] = total;
    for (int i = n; i < MAX_GROUP; ++i) grp.p[i] = grp.p[0];
    grp.n = n;
    if (gs[0].c_f32) return launch_group_tn<false, true>(grp, st);
    return gs[0].accumulate ? launch_group_tn<true, false>(grp, st) : launch_group_tn<false, false>(grp, st);
}

hipError_t gemm_mfma(const GemmArgs &g, hipStream_t st) {
    const int splits = gemm_mfma_splits(g);
    if (splits > 1) {
        GemmP p = params(g);
        p.C = (bf16_t *)g.split_ws; p.ldc = g.N;
        p.accumulate = 0; p.c_f32 = 1;
        p.k_chunk = ceil_div(ceil_div(g.K, splits), BK) * BK;
        p.splits = ceil_div(g.K, p.k_chunk);                          // no empty chunk
        p.split_stride = (long)g.M * g.N;
        hipError_t e = launch_partials(g.layout, p, st);
        if (e != hipSuccess) return e;
        const long quads = ((long)g.M * g.N + 3) / 4;
        if (g.c_f32)
            splitk_reduce_kernel<float><<<ceil_div(quads, 256), 256, 0, st>>>((const float *)g.split_ws, p.splits, p.split_stride,
                                                                            g.M, g.N, (float *)g.C, g.ldc, g.accumulate ? 1 : 0);
        else
            splitk_reduce_kernel<bf16_t><<<ceil_div(quads, 256), 256, 0, st>>>((const float *)g.split_ws, p.splits, p.split_stride,
                                                                             g.M, g.N, (bf16_t *)g.C, g.ldc, g.accumulate ? 1 : 0);
        return hipGetLastError();
    }
    GemmP p = params(g);
    int n_cu = 0, tail_tiles = 0;
    hipError_t e = compute_units(n_cu);
    if (e != hipSuccess) return e;
    const int tail_s = gemm_mfma_tail_splits(g, n_cu, tail_tiles);
    p.tile_count -= tail_tiles;                                       // the full rounds
    if (g.c_f32) e = launch<false, false, false, true>(p, st);
    else {
        const bool add = p.residual || p.accumulate;
        switch (g.layout) {
            case GEMM_NT: e = add ? launch<true, true, true>(p, st) : launch<true, true, false>(p, st); break;
            case GEMM_NN: e = add ? launch<true, false, true>(p, st) : launch<true, false, false>(p, st); break;
            default: e = add ? launch<false, false, true>(p, st) : launch<false, false, false>(p, st); break;
        }
    }
    if (e != hipSuccess || tail_tiles == 0) return e;
    GemmP t = params(g);
    t.C = (bf16_t *)g.split_ws; t.accumulate = 0; t.c_f32 = 1;
    t.tile_begin = p.tile_count; t.tile_count = tail_tiles; t.compact = 1;
    t.k_chunk = ceil_div(ceil_div(g.K, tail_s), BK) * BK;
    t.splits = ceil_div(g.K, t.k_chunk);
    e = launch_partials(g.layout, t, st);
    if (e != hipSuccess) return e;
    if (g.c_f32)
        tail_reduce_kernel<float><<<tail_tiles * 64, 256, 0, st>>>((const float *)g.split_ws, t.splits, t.tile_begin, tail_tiles, t.tiles_m,
                                                                  t.tiles_n, g.M, g.N, (float *)g.C, g.ldc, g.accumulate ? 1 : 0);
    else
        tail_reduce_kernel<bf16_t><<<tail_tiles * 64, 256, 0, st>>>((const float *)g.split_ws, t.splits, t.tile_begin, tail_tiles, t.tiles_m,
                                                                   t.tiles_n, g.M, g.N, (bf16_t *)g.C, g.ldc, g.accumulate ? 1 : 0);
    return hipGetLastError();
}

}  // namespace mmt
