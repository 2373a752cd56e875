// Segment-masked flash attention on the gfx950 matrix cores (bf16 in, fp32 accumulate),
// forward and backward, for packed variable-length segments.
//
// Tiling is on the GLOBAL token index, not per segment: a workgroup owns a run of consecutive queries
// (256 in the forward and dQ kernels, one query per lane of 8 wavefronts; both lane halves of a wavefront
// mirror the same 32 queries) or keys (128 in the dK/dV kernel).  Every query carries its own key range
// [lo, hi) = [segment start, causal ? q + 1 : segment end), so a tile may straddle any number of
// segment boundaries and a pack of many short segments still fills whole tiles.  The key loop of
// a workgroup runs over [lo(first query), hi(last query)) only: tiles that are fully masked for
// the workgroup are never loaded, and 32-key blocks that are fully masked for one wavefront are
// skipped by that wavefront (causal lower triangle, other segments).  The tiles of a launch differ a lot
// in work (a query tile at the end of a long causal segment walks many more keys than one at its start):
// they are dispatched heaviest first, with the head index fastest, from a table the host computes
// (longest-first scheduling as in the paper's Algorithm 1, applied to the GPU's work items).
//
// All score tiles are computed TRANSPOSED (keys x queries): S^T = K . Q^T with the MFMA's row
// operand = keys and column operand = queries.  A lane then holds 16 keys of ONE query per
// 32-key block, so the softmax row reductions are in-lane plus one cross-half exchange, the
// running max / sum / log-sum-exp / D are per-lane scalars, and P^T (or dS^T) is already laid
// out as the column operand of the next MFMA: O^T = V^T . P^T, dQ^T = K^T . dS^T.  The row
// operand of those products is the K or V tile transposed ([feature][key]), its keys in the order in
// which the accumulator registers hold them: all kernels keep the tiles row-major in LDS, as they are copied, and form
// the transposed fragments with the transposing LDS read.
//
// The backward pass is two kernels: dQ (same roles as forward; also writes -D, D = rowsum(dO * O), for the second),
// then dK/dV with one KEY per lane, looping over the query tiles that can see the workgroup's
// keys and over the query heads of the key/value head's group, so grouped-query gradients are
// summed in registers and nothing needs atomics: results are deterministic.  The dK/dV kernel has two forms: for
// heads wider than 64 features a software-pipelined one (one wavefront per SIMD, the next block's scores computed
// under the current block's softmax, whole 64-query steps skipped per wavefront), for 64-wide heads a plain one
// that leaves room for two workgroups per compute unit.
//
// Head dimensions: the kernels are instantiated for 64 and 128 features; a head of another width (a
// multiple of 16, e.g. 80) uses the next instantiation with the missing features read as zero and never
// stored.
#include "kernels.h"
#include <atomic>
#include <algorithm>
#include <type_traits>
#include <utility>

namespace mmt {

namespace {

constexpr int BQ = 128;        // keys per workgroup of the dK/dV kernel
constexpr int END_MASK = 0x3fffffff;
constexpr float LOG2E = 1.4426950408889634f, LN2 = 0.6931471805599453f;

// Swizzle of the 16-byte units of a tile row in LDS: unit u of row `row` stands at position u ^ swz_unit<D>(row).
// What it has to achieve was measured with a microbenchmark of LDS read patterns: a 16-byte-per-lane read is served
// 16 lanes at a time, lanes 0-7 together with 24-31, 8-15 with 16-23 (and the same in the upper half), an 8-byte
// transposing read one 16-lane group at a time, and a group runs at full rate when its lanes fall into distinct 16-byte
// (8-byte) slots modulo 256 bytes.  With 128-byte rows (D = 64) the row's parity supplies one slot bit and a 3-bit
// swizzle does; with 256-byte rows (D = 128) all four unit bits have to come from the swizzle: the fragment reads
// (32 consecutive rows, one unit) need bit 3 to differ between rows 0-7 / 24-31 and 8-15 / 16-23, the transposing
// reads (4 consecutive rows, two neighbouring units) need the row's lowest bit in a unit bit above bit 0.  The
// 3-bit swizzle alone ran both at half rate there.
__device__ __forceinline__ int swz(int row) { return (row ^ (row >> 3)) & 7; }
template <int D>
__device__ __forceinline__ int swz_unit(int row) {
    if constexpr (D == 128) return ((row ^ (row >> 3) ^ ((row & 1) << 2)) & 7) | (((row >> 3) & 1) << 3);
    else return swz(row);
}

__device__ __forceinline__ bf16x8 pack8(const float *v) {
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = (__bf16)v[i];
    return r;
}

__device__ __forceinline__ f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}

#define MFMA(a, b, c) __builtin_amdgcn_mfma_f32_32x32x16_bf16((a), (b), (c), 0, 0, 0)

// The same MFMA written as assembly, with its result in VECTOR registers and its column operand in ACCUMULATION registers.
// In a kernel that needs more than 256 registers the compiler gives every MFMA builtin an accumulation-register result,
// and a result the vector ALU reads next (a score) then costs one copy instruction per element; operands that only MFMAs
// read (a wavefront's own K and V rows) can live in the accumulation half instead.  The compiler does not know what
// these statements are: whoever uses them keeps a result away from the vector ALU until the MFMA has retired
// (mfma_results_settle, or enough other work in between), and never lets two of them in a row depend on each other's result.
__device__ __forceinline__ void mfma_v_first(f32x16 &acc, const bf16x8 &rows, const bf16x8 &cols_acc) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(acc) : "v"(rows), "a"(cols_acc));
}
__device__ __forceinline__ void mfma_v(f32x16 &acc, const bf16x8 &rows, const bf16x8 &cols_acc) {
    asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc) : "v"(rows), "a"(cols_acc));
}
// more wait states than the eight passes of the MFMA above plus its write-back take
__device__ __forceinline__ void mfma_results_settle() { asm volatile("s_nop 15\n\ts_nop 7" ::: "memory"); }


// Per-compute-unit busy time (measurement aid): a workgroup adds its run time, in ticks of the constant 100 MHz
// counter, to the entry of the compute unit it ran on: minus the time at its start, plus the time at its end
// (unsigned wrap-around), so that nothing has to be kept in a register in between.
__device__ __forceinline__ void add_busy(unsigned long long *row, bool end) {
    if (row && threadIdx.x == 0) {
        const unsigned long long t = wall_clock64();
        atomicAdd(row + (__smid() & 1023u), end ? t : 0ull - t);
    }
}

struct RowInfo { int lo, hi; };   // allowed partner range of one token

// Smallest and largest range bounds over the 32 consecutive tokens base .. base + 31 that a wavefront holds one per
// lane (lanes 32 .. 63 repeat them), as scalars.  Both bounds are non-decreasing in the token index (segments follow
// one another in the pack; a causal bound moves with the token), so the first and the last token in range have them.
// No token in range: empty (lo_min = hi_min = INT_MAX, lo_max = hi_max = 0).
struct WaveBounds { int lo_min, lo_max, hi_min, hi_max; };
__device__ __forceinline__ WaveBounds wave_bounds(const RowInfo &me, int base, int T) {
    WaveBounds w = {0x7fffffff, 0, 0x7fffffff, 0};
    const int n = min(T - base, 32);
    if (n > 0) {
        w.lo_min = __builtin_amdgcn_readfirstlane(me.lo);
        w.hi_min = __builtin_amdgcn_readfirstlane(me.hi);
        w.lo_max = __builtin_amdgcn_readlane(me.lo, n - 1);
        w.hi_max = __builtin_amdgcn_readlane(me.hi, n - 1);
    }
    return w;
}

__device__ __forceinline__ RowInfo query_range(const int2 *info, int q, int T) {
    RowInfo r = {0, 0};
    if (q < T) {
        const int2 v = info[q];
        r.lo = v.x;
        r.hi = (v.y >> 30) ? (v.y & END_MASK) : q + 1;
    }
    return r;
}
__device__ __forceinline__ RowInfo key_range(const int2 *info, int k, int T) {
    RowInfo r = {0, 0};
    if (k < T) {
        const int2 v = info[k];
        r.lo = (v.y >> 30) ? v.x : k;
        r.hi = v.y & END_MASK;
    }
    return r;
}

// ------------------------------------------------------------------------------------------
// shared pieces
// ------------------------------------------------------------------------------------------
constexpr int FQ = 256;         // queries per workgroup of the forward and dQ kernels (8 wavefronts x 32)

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((ext_vector_type(4))) uint32_t rawx4;

__device__ __forceinline__ void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

// fragment of a row-major [rows][D] tile (row bytes 2 D): row, k-slice ks (16 features), lane half
template <int D>
__device__ __forceinline__ bf16x8 frag_k(const uint8_t *tile, int row, int ks, int half) {
    constexpr int UPR = D / 8;
    return *reinterpret_cast<const bf16x8 *>(tile + (row * UPR + ((ks * 2 + half) ^ swz_unit<D>(row))) * 16);
}

// ------------------------------------------------------------------------------------------
// backward
// ------------------------------------------------------------------------------------------
// Both backward kernels walk 64-row tiles that are copied global -> LDS directly, row-major ([row][D],
// 16-byte units XOR-swizzled by row), into two slots, the next tile being in flight while the current one
// is multiplied.  A product whose contraction runs over the tile's rows (dQ^T = K^T dS^T, dV^T = dO^T P,
// dK^T = Q^T dS) needs the tile transposed as its row operand; that fragment is formed from the same
// row-major tile by the transposing LDS read (ds_read_b64_tr_b16), with the rows taken in the order in
// which the accumulator registers of the score tile hold them.
constexpr int BT2 = 64;

typedef __attribute__((ext_vector_type(4))) short shortx4;
typedef __attribute__((ext_vector_type(8))) short shortx8;

// One wavefront's share of the copies of [64][D] tiles out of a row-major tensor: N copies of 1 KiB per tile, copy
// (first + i) of a tile covering its rows (first + i) * 512 / D ...  What depends on the lane is computed once
// (init); a copy then costs one addition.  Rows at or beyond the end of the tensor read as zero (the descriptor's
// bounds check), and so do the columns from row_elems on (a head narrower than the tile): their lanes carry an
// offset of 2 GiB, which no tensor reaches (the launchers check), and the sum with the tile's offset cannot wrap.
template <int D, int N>
struct RowCopier {
    static constexpr int UPR = D / 8, ROWS_PER_COPY = 1024 / (2 * D);
    uint32_t off[N];
    int first;
    __device__ __forceinline__ void init(int first_, long ld, int row_elems) {
        first = first_;
        const int lane = threadIdx.x & 63;
        const int lrow = lane / UPR, pos = lane % UPR;
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const int row = (first + i) * ROWS_PER_COPY + lrow;
            const int unit = pos ^ swz_unit<D>(row);
            off[i] = unit * 8 < row_elems ? (uint32_t)((row * ld + unit * 8) * 2) : 0x80000000u;
        }
    }
    // the tile whose first row is row0 and whose first column is col0 of the tensor rs describes (row length ld)
    __device__ __forceinline__ void issue(__amdgpu_buffer_rsrc_t rs, uint8_t *tile, long row0, long ld, long col0) const {
        const uint32_t base = (uint32_t)((row0 * ld + col0) * 2);
#pragma unroll
        for (int i = 0; i < N; ++i)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void *)(tile + (first + i) * ROWS_PER_COPY * 2 * D), 16,
                                                     (int)(off[i] + base), 0, 0, 0);
    }
};
constexpr size_t MAX_TENSOR_BYTES = 0x7fff0000ull;      // what RowCopier's offsets allow

// Transposing reads.  Lane constants: 16-lane group gq = lane >> 4 forms the fragment rows (features)
// 16 (gq & 1) .. + 15 for lane half h = gq >> 1; as a source, lane j = lane & 15 of the group supplies
// the address of tile row 4 h + (j >> 2) (+ a multiple of 8), features 4 (j & 3) .. + 3 of the group's 16.
// tr_off[X] holds that address for each value X of the compile-time part of the swizzled unit position.
template <int D>
struct TrReader {
    uint32_t off[8];
    __device__ __forceinline__ void init(uint32_t lds_base) {
        const int lane = threadIdx.x & 63, gq = lane >> 4, j = lane & 15, qd = j & 3, t = j >> 2, h = gq >> 1;
        // the lane's part of the swizzle of rows 4 h + t (+ a multiple of 8), low three unit bits
        const int L = ((2 * (gq & 1) + (qd >> 1)) ^ swz_unit<D>(4 * h + t)) & 7;
#pragma unroll
        for (int x = 0; x < 8; ++x) off[x] = lds_base + (4 * h + t) * 2 * D + (qd & 1) * 8 + ((x ^ L) << 4);
    }
    // half SEC (elements 4 SEC .. 4 SEC + 3) of the fragment of 32-row block B, MFMA M of the block, feature
    // block C of a tile at byte offset `tile` from lds_base: rows 32 B + 16 M + 8 SEC + 4 h + (0..3)
    template <int B, int M, int C, int SEC>
    __device__ __forceinline__ shortx4 read(uint32_t tile) const {
        constexpr int CST = (4 * B + 2 * M + SEC) & 7, X = (4 * (C & 1)) ^ CST;
        // unit bit 3 (features 64 ..): for 256-byte rows the swizzle flips it in every second group of 8 rows
        constexpr int HI = D == 128 ? ((C >> 1) ^ (SEC & 1)) : (C >> 1);
        constexpr int IMM = (32 * B + 16 * M + 8 * SEC) * 2 * D + HI * 128;
        shortx4 v;
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(off[X] + tile), "n"(IMM));
        return v;
    }
    // the same with the tile's offset already added to the eight addresses (base) and a constant offset on top
    template <int B, int M, int C, int SEC, int EXTRA>
    static __device__ __forceinline__ shortx4 read_at(const uint32_t (&base)[8]) {
        constexpr int CST = (4 * B + 2 * M + SEC) & 7, X = (4 * (C & 1)) ^ CST;
        constexpr int HI = D == 128 ? ((C >> 1) ^ (SEC & 1)) : (C >> 1);
        constexpr int IMM = (32 * B + 16 * M + 8 * SEC) * 2 * D + HI * 128 + EXTRA;
        static_assert(IMM < 65536, "LDS offset field");
        shortx4 v;
        asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(base[X]), "n"(IMM));
        return v;
    }
};
__device__ __forceinline__ bf16x8 join(shortx4 lo, shortx4 hi) {
    const shortx8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return *reinterpret_cast<const bf16x8 *>(&v);
}
// The transposing reads are written as assembly because the compiler makes the builtin wait for every
// direct-to-LDS copy in flight; their results may be used only after this wait, which names them.
#define TR_WAIT4(x) "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3])
#define TR_WAIT2(x) "+v"(x[0]), "+v"(x[1])

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}
typedef __attribute__((address_space(3))) const bf16x8 lds_bf16x8;

// LDS reads of the dK/dV kernel's pipelined section, written as assembly together with their waits: the section
// mixes them with the transposing reads, which the compiler's counting of outstanding LDS operations does not see
// (its waits would come out stricter than needed and undo the look-ahead).  All of them are volatile, so they
// are issued in source order, and LdsSched counts that order.
template <int IMM, typename V>
__device__ __forceinline__ void lds_read16(V &dst, uint32_t addr) {
    static_assert(sizeof(V) == 16 && IMM >= 0 && IMM < 65536, "ds_read_b128");
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(IMM));
}
// x is complete once at most ALLOWED LDS operations issued after its read are outstanding
template <int ALLOWED, typename V>
__device__ __forceinline__ void lds_wait(V &x) {
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(ALLOWED < 15 ? ALLOWED : 15));
}
// Issue order of the section: the log-sum-exps and the D values of the first four queries, PF score fragments;
// then per softmax element e (a chunk): [the fragment of score MFMA e / PER_M + PF] [one transposing read]
// [log-sum-exps and D values of the next four queries, every fourth element].
template <int NM, int PER_M, int PF, int PER_R>
struct LdsSched {
    static constexpr bool has_frag(int e) { return e % PER_M == 0 && e / PER_M + PF < NM; }
    static constexpr bool has_tr(int e) { return e % PER_R == 0; }
    static constexpr int in_chunk(int e) { return (has_frag(e) ? 1 : 0) + (has_tr(e) ? 1 : 0) + ((e & 3) == 0 && (e >> 2) < 3 ? 2 : 0); }
    static constexpr int before(int e) {                 // operations issued before the waits of chunk e
        int n = PF + 2;
        for (int i = 0; i < e; ++i) n += in_chunk(i);
        return n;
    }
    static constexpr int idx_frag(int j) { return j < PF ? 2 + j : before((j - PF) * PER_M); }
    static constexpr int idx_d(int gq) {                 // the later of the two reads for queries 8 gq ..
        return gq == 0 ? 1 : before(4 * (gq - 1)) + (has_frag(4 * (gq - 1)) ? 1 : 0) + (has_tr(4 * (gq - 1)) ? 1 : 0) + 1;
    }
    static constexpr int allowed_frag(int e) { return before(e) - 1 - idx_frag(e / PER_M); }
    static constexpr int allowed_d(int e) { return before(e) - 1 - idx_d(e >> 2); }
};
// 128-wide head (16 score MFMAs, one per element, five fragments ahead, a transposing read per element): in front of
// element 0 seven operations are out; fragment 0 was the third, the first D values the second of them
static_assert(LdsSched<16, 1, 5, 1>::before(0) == 7 && LdsSched<16, 1, 5, 1>::allowed_frag(0) == 4 &&
              LdsSched<16, 1, 5, 1>::allowed_d(0) == 5, "issue order of the pipelined section, start");
// element 0 adds a fragment, a transposing read and two reads for queries 8 .. 11; fragment 1 was the fourth operation
static_assert(LdsSched<16, 1, 5, 1>::before(1) == 11 && LdsSched<16, 1, 5, 1>::allowed_frag(1) == 7 &&
              LdsSched<16, 1, 5, 1>::idx_d(1) == 10 && LdsSched<16, 1, 5, 1>::allowed_d(4) == LdsSched<16, 1, 5, 1>::before(4) - 11,
              "issue order of the pipelined section, first element");

// Inverse rotary embedding of a gradient held in accumulator layout (the backward pass of the rotation that
// was applied to q and k before the attention): feature f < D/2 pairs with f + D/2, which sit in the same
// lane and register index of accumulators c and c + CB/2.  cs = the (cos, sin) row of this lane's token.
template <int CB>
__device__ __forceinline__ void unrotate(f32x16 (&g)[CB], const float2 *cs, int half) {
#pragma unroll
    for (int c = 0; c < CB / 2; ++c)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            const float4 *p4 = reinterpret_cast<const float4 *>(cs + 32 * c + 8 * gq + 4 * half);
            const float4 a = p4[0], b = p4[1];
            const float co[4] = {a.x, a.z, b.x, b.z}, si[4] = {a.y, a.w, b.y, b.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float lo = g[c][4 * gq + e], hi = g[c + CB / 2][4 * gq + e];
                g[c][4 * gq + e] = lo * co[e] + hi * si[e];
                g[c + CB / 2][4 * gq + e] = hi * co[e] - lo * si[e];
            }
        }
}

// Stores a wavefront's 32 x D result (accumulator layout: lane = row, registers = features; 4 consecutive features
// per lane and register quad) as bf16 rows of a row-major tensor.  The rows go through LDS so that a store
// instruction writes 16 bytes per lane and D / 8 lanes cover a row, whole cache lines, instead of 8 bytes into
// each of 32 rows.  stage: STAGE_BYTES<D> bytes of LDS that belong to this wavefront alone and that no wavefront still
// reads as a tile (the callers put a barrier in front).  dst: row 0, feature 0; rows_valid rows and dh features exist.
template <int D>
constexpr int STAGE_BYTES = 32 * (2 * D + 16);
template <int D>
constexpr int ROWS32_BYTES = 32 * D * 2;              // 32 rows of one operand, staged in the tile layout
template <int D>
constexpr int DKV_STAGE_BYTES = 4 * ROWS32_BYTES<D>;  // the pipelined dK/dV kernel's K rows, behind its three slots
template <int D>
constexpr int DQ_LDS_BYTES = 2 * BT2 * D * 2 + 8 * 2 * ROWS32_BYTES<D>;   // the dQ kernel: first slot, then Q and dO rows of 8 wavefronts
template <int D, int CB>
__device__ __forceinline__ void store_rows(uint8_t *stage, const f32x16 (&acc)[CB], float scale, bf16_t *dst, long ld,
                                           int rows_valid, int dh) {
    constexpr int RS = 2 * D + 16, LPR = D / 8, RPI = 64 / LPR;    // row stride in LDS (2-way bank conflicts at most)
    const int lane = threadIdx.x & 63, half = lane >> 5, l32 = lane & 31;
#pragma unroll
    for (int c = 0; c < CB; ++c)
#pragma unroll
        for (int gq = 0; gq < 4; ++gq) {
            uint2 w;
            w.x = pack_bf16x2(acc[c][4 * gq] * scale, acc[c][4 * gq + 1] * scale);
            w.y = pack_bf16x2(acc[c][4 * gq + 2] * scale, acc[c][4 * gq + 3] * scale);
            *reinterpret_cast<uint2 *>(stage + l32 * RS + (32 * c + 8 * gq + 4 * half) * 2) = w;
        }
    const int r0 = lane / LPR, cb = (lane % LPR) * 16;
#pragma unroll
    for (int i = 0; i < 32 / RPI; ++i) {
        const int r = i * RPI + r0;
        const uint4 v = *reinterpret_cast<const uint4 *>(stage + r * RS + cb);
        if (r < rows_valid && cb / 2 < dh) *reinterpret_cast<uint4 *>(dst + (long)r * ld + cb / 2) = v;
    }
}

// ------------------------------------------------------------------------------------------
// backward: dQ (and -D, D = rowsum(dO * O)).  Same roles as the forward kernel: 8 wavefronts x 32 queries.
// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(512) void attn_dq_kernel(AttnArgs a) {
    constexpr int KS = D / 16, CB = D / 32;
    constexpr int TILE = BT2 * D * 2, SLOT = 2 * TILE;             // K tile, then V tile
    constexpr int COPIES = BT2 * D * 2 / 1024 / 4;                 // per wavefront (4 wavefronts per tile)
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    add_busy(a.cu_busy ? a.cu_busy + 1024 : nullptr, false);

    // grid: x = head, y = position in the dispatch order of the query tiles (heaviest first)
    const int head = blockIdx.x, g = head / (a.nh / a.nkv);
    const int q0 = (a.use_order ? a.order_q[blockIdx.y] : blockIdx.y) * FQ;
    // the wavefront's index as a scalar: what is derived from it (copy destinations, buffer descriptors) stays uniform
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), half = lane >> 5, l32 = lane & 31;
    const int T = a.T;
    const bf16_t *qkv = (const bf16_t *)a.qkv;
    const long ld = a.ld_qkv;
    const int dh = a.d;                                 // head dimension in memory (<= D: LDS tiles and fragments are zero-padded to D)
    const int nq = a.nh * dh, nk = a.nkv * dh;

    const int q = q0 + wave * 32 + l32;
    const RowInfo me = query_range(a.tok_info, q, T);
    const bool valid = q < T;
    const WaveBounds wb = wave_bounds(me, q0 + wave * 32, T);
    const int w_lo_min = wb.lo_min, w_lo_max = wb.lo_max, w_hi_max = wb.hi_max, w_hi_min = wb.hi_min;
    const RowInfo first = query_range(a.tok_info, q0, T), last = query_range(a.tok_info, min(q0 + FQ, T) - 1, T);
    const int kbeg = first.lo, kend = last.hi;

    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(qkv), 0, (int)(uint32_t)((size_t)T * ld * 2), 0x00020000);
    // wavefronts 4..7 copy the K tile, wavefronts 0..3 the V tile
    RowCopier<D, COPIES> cp;
    cp.init((wave & 3) * COPIES, ld, dh);
    auto copy_kv = [&](uint8_t *slot, int kt) {
        if (wave >= 4) cp.issue(rs, slot, kt, ld, nq + g * dh);
        else cp.issue(rs, slot + TILE, kt, ld, nq + nk + g * dh);
    };
    TrReader<D> tr;
    tr.init((uint32_t)(uintptr_t)(lds_void *)smem);

    // This wavefront's 32 rows of Q, dO and O: copied into LDS the way tiles are (whole rows per instruction, rows
    // beyond the pack and features beyond the head's width as zeros) and read back in the fragment layout; loading
    // them straight into that layout takes 24 loads of 16 bytes per row and a fifth of the kernel's time on packs
    // of short segments.  They stand behind the first slot (Q and dO side by side, O then in Q's place); the second
    // slot, which they cover, is first written after the first step's barrier.
    bf16x8 qf[KS], dof[KS];
    float Dq = 0.f;
    {
        const __amdgpu_buffer_rsrc_t rs_do = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<bf16_t *>((const bf16_t *)a.d_o), 0, (int)(uint32_t)((size_t)T * nq * 2), 0x00020000);
        const __amdgpu_buffer_rsrc_t rs_o = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<bf16_t *>((const bf16_t *)a.o), 0, (int)(uint32_t)((size_t)T * nq * 2), 0x00020000);
        RowCopier<D, ROWS32_BYTES<D> / 1024> cp_q, cp_o;
        cp_q.init(0, ld, dh);
        cp_o.init(0, nq, dh);
        uint8_t *st_q = smem + SLOT + wave * 2 * ROWS32_BYTES<D>, *st_do = st_q + ROWS32_BYTES<D>;
        cp_q.issue(rs, st_q, q0 + wave * 32, ld, head * dh);
        cp_o.issue(rs_do, st_do, q0 + wave * 32, nq, head * dh);
        copy_kv(smem, kbeg);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            qf[ks] = frag_k<D>(st_q, l32, ks, half);
            dof[ks] = frag_k<D>(st_do, l32, ks, half);
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");           // Q has been read: O may take its place
        cp_o.issue(rs_o, st_q, q0 + wave * 32, nq, head * dh);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 of = frag_k<D>(st_q, l32, ks, half);
            const uint4 w = *reinterpret_cast<const uint4 *>(&dof[ks]), x = *reinterpret_cast<const uint4 *>(&of);
            const uint32_t dw[4] = {w.x, w.y, w.z, w.w}, ow[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                Dq += __uint_as_float(dw[e] << 16) * __uint_as_float(ow[e] << 16);
                Dq += __uint_as_float(dw[e] & 0xffff0000u) * __uint_as_float(ow[e] & 0xffff0000u);
            }
        }
    }
    Dq += __shfl_xor(Dq, 32, 64);
    float lse2 = 0.f;                                  // log-sum-exp in log2 units
    if (valid) {
        lse2 = a.lse[(long)head * T + q] * LOG2E;
        if (half == 0) a.Dsum[(long)head * T + q] = -Dq;                // the dK/dV kernels add it
    }
    // With 64-wide heads dP - D comes out of the matrix core: the dP product of every block starts from -D instead of
    // from zero (a lane holds keys of ONE query, so the 16 accumulator registers of a lane all start from that query's
    // -D).  The 128-wide kernel has no 16 registers to hold that operand and subtracts D element by element.
    constexpr bool D_IN_MFMA = D <= 64;
    f32x16 negD;
#pragma unroll
    for (int i = 0; i < 16; ++i) negD[i] = D_IN_MFMA ? -Dq : 0.f;
    f32x16 dq[CB];
#pragma unroll
    for (int c = 0; c < CB; ++c) dq[c] = zero16();
    const float sl2 = a.scale * LOG2E;

    int slot = 0;
    for (int kt = kbeg; kt < kend; kt += BT2, slot ^= 1) {
        const uint8_t *sK = smem + slot * SLOT, *sV = sK + TILE;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");             // this step's tiles have landed
        lds_barrier();                                               // ... and everyone is done with the other slot
        if (kt + BT2 < kend) copy_kv(smem + (slot ^ 1) * SLOT, kt + BT2);
        auto block = [&](auto B_) {
            constexpr int b = decltype(B_)::value;
            const int kb = kt + 32 * b;
            if (!((kb < w_hi_max) && (kb + 32 > w_lo_min))) return;
            f32x16 s = zero16(), dp = negD;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                s = MFMA(frag_k<D>(sK, 32 * b + l32, ks, half), qf[ks], s);
                dp = MFMA(frag_k<D>(sV, 32 * b + l32, ks, half), dof[ks], dp);
            }
            // K^T fragments of this block: [MFMA m][feature block c], two halves each
            shortx4 t0[4], t1[4], t2[4], t3[4];                      // (m, sec) = (0,0), (0,1), (1,0), (1,1)
            const uint32_t tile = slot * SLOT;
            t0[0] = tr.template read<b, 0, 0, 0>(tile); t1[0] = tr.template read<b, 0, 0, 1>(tile);
            t2[0] = tr.template read<b, 1, 0, 0>(tile); t3[0] = tr.template read<b, 1, 0, 1>(tile);
            t0[1] = tr.template read<b, 0, 1, 0>(tile); t1[1] = tr.template read<b, 0, 1, 1>(tile);
            t2[1] = tr.template read<b, 1, 1, 0>(tile); t3[1] = tr.template read<b, 1, 1, 1>(tile);
            if (CB > 2) {
                t0[2] = tr.template read<b, 0, 2, 0>(tile); t1[2] = tr.template read<b, 0, 2, 1>(tile);
                t2[2] = tr.template read<b, 1, 2, 0>(tile); t3[2] = tr.template read<b, 1, 2, 1>(tile);
                t0[3] = tr.template read<b, 0, 3, 0>(tile); t1[3] = tr.template read<b, 0, 3, 1>(tile);
                t2[3] = tr.template read<b, 1, 3, 0>(tile); t3[3] = tr.template read<b, 1, 3, 1>(tile);
            } else {
                t0[2] = t0[3] = t1[2] = t1[3] = t2[2] = t2[3] = t3[2] = t3[3] = shortx4{0, 0, 0, 0};
            }
            const bool inside = kb >= w_lo_max && kb + 32 <= w_hi_min;
            const unsigned span = (unsigned)(me.hi - me.lo);
            const int rel = kb + 4 * half - me.lo;
            float ds[16];
            // two copies of the loop, so that a block no key of which is masked pays nothing for the mask
            auto softmax = [&](auto MASK_) {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    float p = __builtin_amdgcn_exp2f(fmaf(s[i], sl2, -lse2));
                    if (decltype(MASK_)::value) p = (unsigned)(rel + 8 * (i >> 2) + (i & 3)) < span ? p : 0.f;
                    ds[i] = D_IN_MFMA ? p * dp[i] : p * (dp[i] - Dq);
                }
            };
            if (inside) softmax(std::false_type{});
            else softmax(std::true_type{});
            asm volatile("s_waitcnt lgkmcnt(0)" : TR_WAIT4(t0), TR_WAIT4(t1), TR_WAIT4(t2), TR_WAIT4(t3));
            const bf16x8 ds0 = pack8(ds), ds1 = pack8(ds + 8);
#pragma unroll
            for (int c = 0; c < CB; ++c) {
                dq[c] = MFMA(join(t0[c], t1[c]), ds0, dq[c]);
                dq[c] = MFMA(join(t2[c], t3[c]), ds1, dq[c]);
            }
        };
        block(std::integral_constant<int, 0>{});
        block(std::integral_constant<int, 1>{});
    }
    lds_barrier();                                     // the tiles are done with: LDS now stages the output rows
    if (valid && a.rope_cs) unrotate<CB>(dq, a.rope_cs + (long)q * (D / 2), half);
    store_rows<D, CB>(smem + wave * STAGE_BYTES<D>, dq, a.scale, (bf16_t *)a.d_qkv + (long)(q0 + wave * 32) * ld + head * dh, ld,
                      T - (q0 + wave * 32), dh);
    add_busy(a.cu_busy ? a.cu_busy + 1024 : nullptr, true);
}

// Exchange between lane l and lane l ^ 32 in one vector instruction (the two halves of a wavefront hold the two halves of
// every query's keys): after the swap the first result holds the lower half's values in both halves, the second the upper's.
__device__ __forceinline__ float max_across_halves(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float sum_across_halves(float v) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}
// The forward kernel's running maximum is lazy: the reference the exponentials are taken against moves only when a
// step's maximum exceeds it by more than 2^LAZY_LOG2 (in units of the exponent), so the output accumulators are rescaled
// a few times per query instead of at almost every step; exponentials stay below 2^LAZY_LOG2, far inside fp32 and bf16 range.
constexpr float LAZY_LOG2 = 8.f;

// ------------------------------------------------------------------------------------------
// forward.  WAVES wavefronts x 32 queries per workgroup, two wavefronts per SIMD either way (so that one can run its
// softmax on the vector ALUs while the other occupies the matrix core): 8 wavefronts = 256 queries, one workgroup per
// compute unit (every K / V tile is fetched once for 256 queries), or 4 wavefronts = 128 queries, two workgroups per
// compute unit (less masked work on short segments; used for 64-wide heads).  The keys are walked 64 at a time through
// two LDS slots of {K tile, V tile}, both copied global -> LDS directly in their memory order (wavefronts 4..7 copy K,
// 0..3 copy V).  O^T = V^T . P^T takes V^T from the row-major tile by the transposing LDS read, the same scheme as
// dQ^T = K^T . dS^T above.  One barrier per step: after it every wavefront has finished the previous step, so the slot
// that step used may be refilled.
// ------------------------------------------------------------------------------------------
template <int D, int WAVES>
__global__ __launch_bounds__(WAVES * 64, 2) void attn_fwd_kernel(AttnArgs a) {
    constexpr int FQW = WAVES * 32;                                // queries per workgroup
    constexpr int KS = D / 16, CB = D / 32;
    constexpr int TILE = BT2 * D * 2, SLOT = 2 * TILE;             // K tile, then V tile
    constexpr int COPIES = BT2 * D * 2 / 1024 / 4;                 // per wavefront and tile (four wavefronts copy a tile)
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    const int head = blockIdx.x, g = head / (a.nh / a.nkv);
    // the dispatch order is kept per FQ-query tile; the workgroups of one tile (two, with four wavefronts each) follow each other
    constexpr int PER_TILE = FQ / FQW;
    const int q0 = (a.use_order ? a.order_q[blockIdx.y / PER_TILE] * PER_TILE + blockIdx.y % PER_TILE : blockIdx.y) * FQW;
    if (q0 >= a.T) return;                                         // second half of a last tile that the pack only half fills
    add_busy(a.cu_busy, false);
    // the wavefront's index as a scalar: what is derived from it (copy destinations, buffer descriptors) stays uniform
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), half = lane >> 5, l32 = lane & 31;
    const int T = a.T;
    const bf16_t *qkv = (const bf16_t *)a.qkv;
    const long ld = a.ld_qkv;
    const int dh = a.d;
    const int nq = a.nh * dh, nk = a.nkv * dh;

    const int q = q0 + wave * 32 + l32;
    const RowInfo me = query_range(a.tok_info, q, T);
    const bool valid = q < T;
    const WaveBounds wb = wave_bounds(me, q0 + wave * 32, T);
    const int w_lo_min = wb.lo_min, w_lo_max = wb.lo_max, w_hi_max = wb.hi_max, w_hi_min = wb.hi_min;
    const RowInfo first = query_range(a.tok_info, q0, T), last = query_range(a.tok_info, min(q0 + FQW, T) - 1, T);
    const int kbeg = first.lo, kend = last.hi;

    bf16x8 qf[KS];                                     // this wavefront's Q rows as the MFMA's column operand (filled below)
    f32x16 oacc[CB];
#pragma unroll
    for (int c = 0; c < CB; ++c) oacc[c] = zero16();
    float m_run = -INFINITY, l_run = 0.f;
    const float sl2 = a.scale * LOG2E;

    const __amdgpu_buffer_rsrc_t rs =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(qkv), 0, (int)(uint32_t)((size_t)T * ld * 2), 0x00020000);
    // eight wavefronts: 4..7 copy the K tile, 0..3 the V tile; four wavefronts: each copies its quarter of both
    RowCopier<D, COPIES> cp;
    cp.init((wave & 3) * COPIES, ld, dh);
    auto copy_kv = [&](uint8_t *slot, int kt) {
        if (WAVES == 4 || wave >= 4) cp.issue(rs, slot, kt, ld, nq + g * dh);
        if (WAVES == 4 || wave < 4) cp.issue(rs, slot + TILE, kt, ld, nq + nk + g * dh);
    };
    TrReader<D> tr;
    tr.init((uint32_t)(uintptr_t)(lds_void *)smem);

    // The Q rows go through LDS like the dQ kernel's Q, dO and O rows (see there): behind the two slots, or, with four
    // wavefronts (whose Q rows fill a slot exactly), in the second slot, which is first written after the first barrier.
    {
        RowCopier<D, ROWS32_BYTES<D> / 1024> cp_q;
        cp_q.init(0, ld, dh);
        uint8_t *st_q = smem + (WAVES == 4 ? SLOT : 2 * SLOT) + wave * ROWS32_BYTES<D>;
        cp_q.issue(rs, st_q, q0 + wave * 32, ld, head * dh);
        copy_kv(smem, kbeg);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[ks] = frag_k<D>(st_q, l32, ks, half);
    }
    int slot = 0;
    for (int kt = kbeg; kt < kend; kt += BT2, slot ^= 1) {
        const uint8_t *sK = smem + slot * SLOT;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");             // this step's tiles have landed
        lds_barrier();                                               // ... and everyone is done with the other slot
        if (kt + BT2 < kend) copy_kv(smem + (slot ^ 1) * SLOT, kt + BT2);
        bool act[2];
#pragma unroll
        for (int b = 0; b < 2; ++b) act[b] = (kt + 32 * b < w_hi_max) && (kt + 32 * b + 32 > w_lo_min);
        if (!(act[0] || act[1])) continue;
        f32x16 s[2];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            s[b] = zero16();
            if (act[b]) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) s[b] = MFMA(frag_k<D>(sK, 32 * b + l32, ks, half), qf[ks], s[b]);
            }
        }
        // online softmax on the raw scores (the scale is folded into the exponent);
        // register i of block b  <->  key kt + 32 b + 8 (i >> 2) + 4 half + (i & 3)
        float mx = -INFINITY;
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            if (!act[b]) continue;
            const int kb = kt + 32 * b;
            if (!(kb >= w_lo_max && kb + 32 <= w_hi_min)) {            // some lane needs masking
                const unsigned span = (unsigned)(me.hi - me.lo);
                const int rel = kb + 4 * half - me.lo;
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    s[b][i] = (unsigned)(rel + 8 * (i >> 2) + (i & 3)) < span ? s[b][i] : -INFINITY;
            }
#pragma unroll
            for (int i = 0; i < 16; ++i) mx = fmaxf(mx, s[b][i]);
        }
        mx = max_across_halves(mx);
        // move the reference only where the step's maximum is more than 2^LAZY_LOG2 above it (always from -inf)
        const bool need = (mx - m_run) * sl2 > LAZY_LOG2;
        if (__builtin_amdgcn_ballot_w64(need) != 0) {
            const float corr = need ? __builtin_amdgcn_exp2f((m_run - mx) * sl2) : 1.f;
            m_run = need ? mx : m_run;
            l_run *= corr;
#pragma unroll
            for (int c = 0; c < CB; ++c)
#pragma unroll
                for (int i = 0; i < 16; ++i) oacc[c][i] *= corr;
        }
        const float msc = m_run == -INFINITY ? 0.f : m_run * sl2;
        const uint32_t tv = slot * SLOT + TILE;
        auto block = [&](auto B_) {
            constexpr int b = decltype(B_)::value;
            if (!act[b]) return;
            // V^T fragments of this block: [MFMA m][feature block c], two halves each; in flight during the exponentials
            shortx4 t0[4], t1[4], t2[4], t3[4];
            t0[0] = tr.template read<b, 0, 0, 0>(tv); t1[0] = tr.template read<b, 0, 0, 1>(tv);
            t2[0] = tr.template read<b, 1, 0, 0>(tv); t3[0] = tr.template read<b, 1, 0, 1>(tv);
            t0[1] = tr.template read<b, 0, 1, 0>(tv); t1[1] = tr.template read<b, 0, 1, 1>(tv);
            t2[1] = tr.template read<b, 1, 1, 0>(tv); t3[1] = tr.template read<b, 1, 1, 1>(tv);
            if (CB > 2) {
                t0[2] = tr.template read<b, 0, 2, 0>(tv); t1[2] = tr.template read<b, 0, 2, 1>(tv);
                t2[2] = tr.template read<b, 1, 2, 0>(tv); t3[2] = tr.template read<b, 1, 2, 1>(tv);
                t0[3] = tr.template read<b, 0, 3, 0>(tv); t1[3] = tr.template read<b, 0, 3, 1>(tv);
                t2[3] = tr.template read<b, 1, 3, 0>(tv); t3[3] = tr.template read<b, 1, 3, 1>(tv);
            } else {
                t0[2] = t0[3] = t1[2] = t1[3] = t2[2] = t2[3] = t3[2] = t3[3] = shortx4{0, 0, 0, 0};
            }
            float p[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                p[i] = __builtin_amdgcn_exp2f(fmaf(s[b][i], sl2, -msc));
                l_run += p[i];
            }
            asm volatile("s_waitcnt lgkmcnt(0)" : TR_WAIT4(t0), TR_WAIT4(t1), TR_WAIT4(t2), TR_WAIT4(t3));
            const bf16x8 p0 = pack8(p), p1 = pack8(p + 8);
#pragma unroll
            for (int c = 0; c < CB; ++c) {
                oacc[c] = MFMA(join(t0[c], t1[c]), p0, oacc[c]);
                oacc[c] = MFMA(join(t2[c], t3[c]), p1, oacc[c]);
            }
        };
        block(std::integral_constant<int, 0>{});
        block(std::integral_constant<int, 1>{});
    }

    const float l_tot = sum_across_halves(l_run);
    lds_barrier();                                     // the tiles are done with: LDS now stages the output rows
    store_rows<D, CB>(smem + wave * STAGE_BYTES<D>, oacc, valid ? 1.f / l_tot : 0.f, (bf16_t *)a.o + (long)(q0 + wave * 32) * nq + head * dh,
                      nq, T - (q0 + wave * 32), dh);
    if (valid && half == 0) a.lse[(long)head * T + q] = (m_run * sl2 + __builtin_amdgcn_logf(l_tot)) * LN2;
    add_busy(a.cu_busy, true);
}

// ------------------------------------------------------------------------------------------
// backward: dK, dV.  One key per lane (4 wavefronts x 32 keys); loop over the query heads of the group and
// over the 64-query tiles that can see the workgroup's keys.
// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_dkv_kernel(AttnArgs a) {
    constexpr int KS = D / 16, CB = D / 32;
    constexpr int TILE = BT2 * D * 2, SLOT = 2 * TILE + 2 * BT2 * 4;   // Q tile, dO tile, lse[64], D[64]
    constexpr int COPIES = BT2 * D * 2 / 1024 / 4;                     // per wavefront and tile
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    add_busy(a.cu_busy ? a.cu_busy + 2048 : nullptr, false);

    // grid: x = key/value head, y = position in the dispatch order of the key tiles (heaviest first)
    const int g = blockIdx.x, group = a.nh / a.nkv;
    const int k0 = (a.use_order ? a.order_k[blockIdx.y] : blockIdx.y) * BQ;
    // the wavefront's index as a scalar: what is derived from it (copy destinations, buffer descriptors) stays uniform
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), half = lane >> 5, l32 = lane & 31;
    const int T = a.T;
    const bf16_t *qkv = (const bf16_t *)a.qkv;
    const bf16_t *dO = (const bf16_t *)a.d_o;
    const long ld = a.ld_qkv;
    const int dh = a.d;                                 // head dimension in memory (<= D: LDS tiles and fragments are zero-padded to D)
    const int nq = a.nh * dh, nk = a.nkv * dh;

    const int key = k0 + wave * 32 + l32;
    const RowInfo me = key_range(a.tok_info, key, T);       // queries [lo, hi) see this key
    const bool valid = key < T;
    const WaveBounds wb = wave_bounds(me, k0 + wave * 32, T);
    const int w_lo_min = wb.lo_min, w_lo_max = wb.lo_max, w_hi_max = wb.hi_max, w_hi_min = wb.hi_min;
    const RowInfo first = key_range(a.tok_info, k0, T), last = key_range(a.tok_info, min(k0 + BQ, T) - 1, T);
    const int qbeg = first.lo, qend = last.hi;

    bf16x8 kf[KS], vf[KS];                             // this wavefront's K and V rows as MFMA operands (filled below)
    f32x16 dk[CB], dv[CB];
#pragma unroll
    for (int c = 0; c < CB; ++c) { dk[c] = zero16(); dv[c] = zero16(); }
    const float sl2 = a.scale * LOG2E;

    const __amdgpu_buffer_rsrc_t rs_q =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(qkv), 0, (int)(uint32_t)((size_t)T * ld * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_do =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(dO), 0, (int)(uint32_t)((size_t)T * nq * 2), 0x00020000);
    // every wavefront copies a quarter of the Q tile and of the dO tile; wavefronts 0 and 1 also fetch the
    // 64 log-sum-exps and the 64 D values of the tile's queries (4 bytes per lane; queries >= T read as 0)
    RowCopier<D, COPIES> cp_q, cp_do;
    cp_q.init(wave * COPIES, ld, dh);
    cp_do.init(wave * COPIES, nq, dh);
    auto copy_tile = [&](uint8_t *slot, int head, int qt) {
        cp_q.issue(rs_q, slot, qt, ld, head * dh);
        cp_do.issue(rs_do, slot + TILE, qt, nq, head * dh);
        if (wave < 2) {
            const float *src = (wave == 0 ? a.lse : a.Dsum) + (long)head * T;
            const __amdgpu_buffer_rsrc_t rs_f =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(src), 0, (int)(uint32_t)((size_t)T * 4), 0x00020000);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_f, (lds_void *)(slot + 2 * TILE + wave * BT2 * 4), 4,
                                                     (int)((qt + lane) * 4), 0, 0, 0);
        }
    };
    TrReader<D> tr;
    tr.init((uint32_t)(uintptr_t)(lds_void *)smem);

    if (qbeg >= qend) goto done;      // no query sees these keys (cannot happen for a key of a segment: it sees itself)
    {
    // The (head, query tile) pairs form one sequence of steps, every step two blocks of 32 queries.  The blocks are
    // software-pipelined: while the vector ALU turns the scores of a block into P and dS, the matrix core computes
    // the scores of the block after it (one MFMA in front of every element of the softmax, so that neither unit
    // waits for the other in this one-wavefront-per-SIMD kernel); the dV and dK products of the block follow.
    // Three LDS slots: a step's second block reads the next step's tile for its look-ahead scores, so the copy of
    // tile step + 2 is issued at the barrier in the middle of step `step`, into the slot tile step - 1 has left.
    // A wavefront skips the steps none of whose queries sees any of its keys; the scores behind such a gap are
    // computed on their own.
    const int tiles_per_head = (qend - qbeg + BT2 - 1) / BT2, n_steps = group * tiles_per_head;
    auto head_of = [&](int step) { return g * group + step / tiles_per_head; };
    auto qt_of = [&](int step) { return qbeg + (step % tiles_per_head) * BT2; };
    const unsigned span = (unsigned)(me.hi - me.lo);

    // LDS addresses, shared by all blocks.  A fragment of the score MFMAs: row 32 bn + l32 of a tile, 16-byte unit
    // (2 ks + half) ^ swz_unit(row), and swz_unit(32 + l32) = swz_unit(l32) ^ 4, so block 1 finds slice ks where block 0
    // finds slice ks ^ 2, 32 rows further on.
    uint32_t f0[KS];
#pragma unroll
    for (int k = 0; k < KS; ++k)
        f0[k] = (uint32_t)(uintptr_t)(lds_void *)smem + (l32 * (D / 8) + ((2 * k + half) ^ swz_unit<D>(l32))) * 16;
    const uint32_t l0 = (uint32_t)(uintptr_t)(lds_void *)smem + 2 * TILE + half * 16;
    uint32_t fcur[KS], fnxt[KS], trc[8], lcur = 0;    // ... of the current step's tile, of the next step's
    int qt_cur = 0;
    int mbase = 0;                                      // first query of this lane's quads minus the first that sees its key
    f32x16 sc[2], dpc[2];                               // scores and dP of a step's two blocks

    auto score_frag = [&](const uint32_t (&fa)[KS], auto BN_, auto J_) -> bf16x8 {
        constexpr int bn = decltype(BN_)::value, j = decltype(J_)::value, ks = j >> 1;
        return *(lds_bf16x8 *)(uintptr_t)(fa[ks ^ (2 * bn)] + ((j & 1) * TILE + bn * 64 * D));
    };
    auto issue_frag = [&](bf16x8 &dst, const uint32_t (&fa)[KS], auto BN_, auto J_) {
        constexpr int bn = decltype(BN_)::value, j = decltype(J_)::value, ks = j >> 1;
        lds_read16<(j & 1) * TILE + bn * 64 * D>(dst, fa[ks ^ (2 * bn)]);
    };
    // the scores of block 0 of the current tile, on their own
    auto scores0 = [&]() {
        static_for<0, 2 * KS>([&](auto J_) {
            constexpr int j = decltype(J_)::value;
            const bf16x8 f = score_frag(fcur, std::integral_constant<int, 0>{}, J_);
            if constexpr (j == 0) mfma_v_first(sc[0], f, kf[0]);
            else if constexpr (j == 1) mfma_v_first(dpc[0], f, vf[0]);
            else if constexpr ((j & 1) == 0) mfma_v(sc[0], f, kf[j >> 1]);
            else mfma_v(dpc[0], f, vf[j >> 1]);
        });
        mfma_results_settle();                         // the softmax reads them next
    };
    // block b of the current tile: softmax from (sc[b], dpc[b]) with the look-ahead scores of the block after it into
    // (sc[b ^ 1], dpc[b ^ 1]), then dV += dO^T P and dK += Q^T dS
    auto block = [&](auto B_) {
        constexpr int b = decltype(B_)::value;
        constexpr int NM = 2 * KS, PER_M = 16 / NM, PF = NM > 8 ? 5 : 3;          // score MFMAs, softmax elements per MFMA, fragments in flight
        constexpr int NR = 4 * CB, PER_R = 16 / NR;                  // transposing reads of the block's first 16 queries
        const uint32_t (&fa)[KS] = b == 0 ? fcur : fnxt;
        constexpr std::integral_constant<int, b ^ 1> BN{};
        shortx4 o0[CB], o1[CB], q0f[CB], q1f[CB], o2[CB], o3[CB], q2f[CB], q3f[CB];
        uint32_t pp[8], dd[8];
        auto fused = [&](auto MASK_) {
            constexpr bool MASK = decltype(MASK_)::value;
            using Sched = LdsSched<NM, PER_M, PF, PER_R>;
            bf16x8 fr[NM];
            f32x4 l4[4], d4[4];
            lds_read16<b * 128>(l4[0], lcur);
            lds_read16<b * 128 + BT2 * 4>(d4[0], lcur);
            static_for<0, PF>([&](auto J_) { issue_frag(fr[decltype(J_)::value], fa, BN, J_); });
            __builtin_amdgcn_sched_barrier(0);         // (the first reads stay in front of the elements' chunks)
            float pprev = 0.f, dprev = 0.f;
            static_for<0, 16>([&](auto E_) {
                constexpr int e = decltype(E_)::value, gq = e >> 2, el = e & 3;
                if constexpr (el == 0) { lds_wait<Sched::allowed_d(e)>(l4[gq]); lds_wait<Sched::allowed_d(e)>(d4[gq]); }
                if constexpr (e % PER_M == 0) {
                    constexpr int j = e / PER_M;
                    lds_wait<Sched::allowed_frag(e)>(fr[j]);
                    // (the vector ALU reads these results no earlier than the next block's softmax, behind this block's
                    // 4 CB dV / dK products; the two chains alternate, so no MFMA follows the one whose result it adds to)
                    if constexpr (j == 0) mfma_v_first(sc[b ^ 1], fr[j], kf[0]);
                    else if constexpr (j == 1) mfma_v_first(dpc[b ^ 1], fr[j], vf[0]);
                    else if constexpr ((j & 1) == 0) mfma_v(sc[b ^ 1], fr[j], kf[j >> 1]);
                    else mfma_v(dpc[b ^ 1], fr[j], vf[j >> 1]);
                    if constexpr (j + PF < NM) issue_frag(fr[j + PF], fa, BN, std::integral_constant<int, j + PF>{});
                }
                if constexpr (e % PER_R == 0) {                      // read r: feature block r / 4; dO or Q; first or second quad
                    constexpr int r = e / PER_R, c = r >> 2;
                    if constexpr ((r & 3) == 0) o0[c] = TrReader<D>::template read_at<b, 0, c, 0, TILE>(trc);
                    if constexpr ((r & 3) == 1) o1[c] = TrReader<D>::template read_at<b, 0, c, 1, TILE>(trc);
                    if constexpr ((r & 3) == 2) q0f[c] = TrReader<D>::template read_at<b, 0, c, 0, 0>(trc);
                    if constexpr ((r & 3) == 3) q1f[c] = TrReader<D>::template read_at<b, 0, c, 1, 0>(trc);
                }
                if constexpr (el == 0 && gq < 3) {
                    lds_read16<b * 128 + (gq + 1) * 32>(l4[gq + 1], lcur);
                    lds_read16<b * 128 + (gq + 1) * 32 + BT2 * 4>(d4[gq + 1], lcur);
                }
                const float lv = l4[gq][el], dvv = d4[gq][el];
                float pv = __builtin_amdgcn_exp2f(fmaf(sc[b][e], sl2, -lv * LOG2E));
                if (MASK) pv = (unsigned)(mbase + (32 * b + 8 * gq + el)) < span ? pv : 0.f;
                const float dsv = pv * (dpc[b][e] + dvv);           // the D array holds -D
                if constexpr (e & 1) { pp[e >> 1] = pack_bf16x2(pprev, pv); dd[e >> 1] = pack_bf16x2(dprev, dsv); }
                else { pprev = pv; dprev = dsv; }
                __builtin_amdgcn_sched_barrier(0);
            });
        };
        if (qt_cur + 32 * b >= w_lo_max && qt_cur + 32 * b + 32 <= w_hi_min) fused(std::false_type{});
        else fused(std::true_type{});
        auto frag4 = [](const uint32_t *w) {
            const uint4 v = make_uint4(w[0], w[1], w[2], w[3]);
            return *reinterpret_cast<const bf16x8 *>(&v);
        };
        if constexpr (CB > 2) asm volatile("s_waitcnt lgkmcnt(0)" : TR_WAIT4(o0), TR_WAIT4(o1), TR_WAIT4(q0f), TR_WAIT4(q1f));
        else asm volatile("s_waitcnt lgkmcnt(0)" : TR_WAIT2(o0), TR_WAIT2(o1), TR_WAIT2(q0f), TR_WAIT2(q1f));
        static_for<0, CB>([&](auto C_) {                             // in flight during the next 2 CB MFMAs
            constexpr int c = decltype(C_)::value;
            o2[c] = TrReader<D>::template read_at<b, 1, c, 0, TILE>(trc); o3[c] = TrReader<D>::template read_at<b, 1, c, 1, TILE>(trc);
            q2f[c] = TrReader<D>::template read_at<b, 1, c, 0, 0>(trc); q3f[c] = TrReader<D>::template read_at<b, 1, c, 1, 0>(trc);
        });
        {
            const bf16x8 pf = frag4(pp), dsf = frag4(dd);
#pragma unroll
            for (int c = 0; c < CB; ++c) {
                dv[c] = MFMA(join(o0[c], o1[c]), pf, dv[c]);
                dk[c] = MFMA(join(q0f[c], q1f[c]), dsf, dk[c]);
            }
        }
        if constexpr (CB > 2) asm volatile("s_waitcnt lgkmcnt(0)" : TR_WAIT4(o2), TR_WAIT4(o3), TR_WAIT4(q2f), TR_WAIT4(q3f));
        else asm volatile("s_waitcnt lgkmcnt(0)" : TR_WAIT2(o2), TR_WAIT2(o3), TR_WAIT2(q2f), TR_WAIT2(q3f));
        {
            const bf16x8 pf = frag4(pp + 4), dsf = frag4(dd + 4);
#pragma unroll
            for (int c = 0; c < CB; ++c) {
                dv[c] = MFMA(join(o2[c], o3[c]), pf, dv[c]);
                dk[c] = MFMA(join(q2f[c], q3f[c]), dsf, dk[c]);
            }
        }
    };

    // K and V rows of this wavefront's 32 keys: copied into LDS the way tiles are (whole rows per instruction, rows
    // beyond the pack and features beyond the head's width as zeros) and read back as fragments; loading them
    // straight into the fragment layout takes 16 loads of 16 bytes per row.  The V rows stand in the third slot, which
    // the barrier below frees for the third tile, the K rows behind the slots.
    {
        constexpr int HALF_TILE = 32 * D * 2;
        static_assert(4 * HALF_TILE <= SLOT && DKV_STAGE_BYTES<D> == 4 * HALF_TILE, "room for the staged K and V rows");
        RowCopier<D, HALF_TILE / 1024> cp_kv;
        cp_kv.init(0, ld, dh);
        uint8_t *stage_k = smem + 3 * SLOT + wave * HALF_TILE, *stage_v = smem + 2 * SLOT + wave * HALF_TILE;
        cp_kv.issue(rs_q, stage_k, k0 + wave * 32, ld, nq + g * dh);
        cp_kv.issue(rs_q, stage_v, k0 + wave * 32, ld, nq + nk + g * dh);
        copy_tile(smem, head_of(0), qt_of(0));
        if (n_steps > 1) copy_tile(smem + SLOT, head_of(1), qt_of(1));
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            kf[ks] = frag_k<D>(stage_k, l32, ks, half);
            vf[ks] = frag_k<D>(stage_v, l32, ks, half);
        }
    }
    lds_barrier();
    int slot = 0;
    bool have0 = false;                                // block 0's scores of this step were computed by the step before
    for (int step = 0; step < n_steps; ++step) {
        const int qt = qt_of(step), nslot = slot == 2 ? 0 : slot + 1;
        qt_cur = qt;
        const bool more = step + 1 < n_steps;
        const bool act = qt < w_hi_max && qt + BT2 > w_lo_min;
        if (act) {
#pragma unroll
            for (int k = 0; k < KS; ++k) { fcur[k] = f0[k] + slot * SLOT; fnxt[k] = f0[k] + nslot * SLOT; }
#pragma unroll
            for (int x = 0; x < 8; ++x) trc[x] = tr.off[x] + slot * SLOT;
            lcur = l0 + slot * SLOT;
            mbase = qt + 4 * half - me.lo;
            if (!have0) scores0();
            block(std::integral_constant<int, 0>{});
        }
        if (more) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");         // the next step's tile has landed
            lds_barrier();                                           // ... for everyone, and tile step - 1 is no longer read
            if (step + 2 < n_steps) copy_tile(smem + (nslot == 2 ? 0 : nslot + 1) * SLOT, head_of(step + 2), qt_of(step + 2));
        }
        if (act) block(std::integral_constant<int, 1>{});
        have0 = act;
        slot = nslot;
    }
    }
done:
    lds_barrier();                                     // the tiles are done with: LDS now stages the output rows
    {
        bf16_t *okp = (bf16_t *)a.d_qkv + (long)(k0 + wave * 32) * ld + nq + g * dh;
        uint8_t *stage = smem + wave * STAGE_BYTES<D>;
        store_rows<D, CB>(stage, dv, 1.f, okp + nk, ld, T - (k0 + wave * 32), dh);
        if (valid && a.rope_cs) unrotate<CB>(dk, a.rope_cs + (long)key * (D / 2), half);
        store_rows<D, CB>(stage, dk, a.scale, okp, ld, T - (k0 + wave * 32), dh);
    }
    add_busy(a.cu_busy ? a.cu_busy + 2048 : nullptr, true);
}

// ------------------------------------------------------------------------------------------
// backward: dK, dV, the plain form: a block's scores, its softmax and its products one after the other, two LDS
// slots.  Used for the 64-wide head, where it fits 256 registers, so that two workgroups share a compute unit
// and overlap each other's phases; the pipelined kernel above needs more registers than that at any width.
// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void attn_dkv_plain_kernel(AttnArgs a) {
    constexpr int KS = D / 16, CB = D / 32;
    constexpr int TILE = BT2 * D * 2, SLOT = 2 * TILE + 2 * BT2 * 4;   // Q tile, dO tile, lse[64], D[64]
    constexpr int COPIES = BT2 * D * 2 / 1024 / 4;                     // per wavefront and tile
    extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
    add_busy(a.cu_busy ? a.cu_busy + 2048 : nullptr, false);

    // grid: x = key/value head, y = position in the dispatch order of the key tiles (heaviest first)
    const int g = blockIdx.x, group = a.nh / a.nkv;
    const int k0 = (a.use_order ? a.order_k[blockIdx.y] : blockIdx.y) * BQ;
    // the wavefront's index as a scalar: what is derived from it (copy destinations, buffer descriptors) stays uniform
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), half = lane >> 5, l32 = lane & 31;
    const int T = a.T;
    const bf16_t *qkv = (const bf16_t *)a.qkv;
    const bf16_t *dO = (const bf16_t *)a.d_o;
    const long ld = a.ld_qkv;
    const int dh = a.d;                                 // head dimension in memory (<= D: LDS tiles and fragments are zero-padded to D)
    const int nq = a.nh * dh, nk = a.nkv * dh;

    const int key = k0 + wave * 32 + l32;
    const RowInfo me = key_range(a.tok_info, key, T);       // queries [lo, hi) see this key
    const bool valid = key < T;
    const WaveBounds wb = wave_bounds(me, k0 + wave * 32, T);
    const int w_lo_min = wb.lo_min, w_lo_max = wb.lo_max, w_hi_max = wb.hi_max, w_hi_min = wb.hi_min;
    const RowInfo first = key_range(a.tok_info, k0, T), last = key_range(a.tok_info, min(k0 + BQ, T) - 1, T);
    const int qbeg = first.lo, qend = last.hi;

    bf16x8 kf[KS], vf[KS];                             // this wavefront's K and V rows as MFMA operands (filled below)
    f32x16 dk[CB], dv[CB];
#pragma unroll
    for (int c = 0; c < CB; ++c) { dk[c] = zero16(); dv[c] = zero16(); }
    const float sl2 = a.scale * LOG2E;

    const __amdgpu_buffer_rsrc_t rs_q =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(qkv), 0, (int)(uint32_t)((size_t)T * ld * 2), 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_do =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t *>(dO), 0, (int)(uint32_t)((size_t)T * nq * 2), 0x00020000);
    // every wavefront copies a quarter of the Q tile and of the dO tile; wavefronts 0 and 1 also fetch the
    // 64 log-sum-exps and the 64 D values of the tile's queries (4 bytes per lane; queries >= T read as 0)
    RowCopier<D, COPIES> cp_q, cp_do;
    cp_q.init(wave * COPIES, ld, dh);
    cp_do.init(wave * COPIES, nq, dh);
    auto copy_tile = [&](uint8_t *slot, int head, int qt) {
        cp_q.issue(rs_q, slot, qt, ld, head * dh);
        cp_do.issue(rs_do, slot + TILE, qt, nq, head * dh);
        if (wave < 2) {
            const float *src = (wave == 0 ? a.lse : a.Dsum) + (long)head * T;
            const __amdgpu_buffer_rsrc_t rs_f =
                __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(src), 0, (int)(uint32_t)((size_t)T * 4), 0x00020000);
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_f, (lds_void *)(slot + 2 * TILE + wave * BT2 * 4), 4,
                                                     (int)((qt + lane) * 4), 0, 0, 0);
        }
    };
    TrReader<D> tr;
    tr.init((uint32_t)(uintptr_t)(lds_void *)smem);

    if (qbeg >= qend) goto done;      // no query sees these keys (cannot happen for a key of a segment: it sees itself)
    {
    // the (head, query tile) pairs form one sequence; the copy of the next pair is in flight during this one
    const int tiles_per_head = (qend - qbeg + BT2 - 1) / BT2, n_steps = group * tiles_per_head;
    // the K and V rows go through LDS as in the pipelined kernel, behind the two slots
    {
        RowCopier<D, ROWS32_BYTES<D> / 1024> cp_kv;
        cp_kv.init(0, ld, dh);
        uint8_t *stage_k = smem + 2 * SLOT + wave * 2 * ROWS32_BYTES<D>, *stage_v = stage_k + ROWS32_BYTES<D>;
        cp_kv.issue(rs_q, stage_k, k0 + wave * 32, ld, nq + g * dh);
        cp_kv.issue(rs_q, stage_v, k0 + wave * 32, ld, nq + nk + g * dh);
        copy_tile(smem, g * group, qbeg);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            kf[ks] = frag_k<D>(stage_k, l32, ks, half);
            vf[ks] = frag_k<D>(stage_v, l32, ks, half);
        }
    }
    int slot = 0;
    for (int step = 0; step < n_steps; ++step, slot ^= 1) {
        const int hh = step / tiles_per_head, qt = qbeg + (step % tiles_per_head) * BT2;
        const uint8_t *sQ = smem + slot * SLOT, *sdO = sQ + TILE;
        const float *sLse = reinterpret_cast<const float *>(sQ + 2 * TILE), *sD = sLse + BT2;
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");             // this step's tiles have landed
        lds_barrier();                                               // ... and everyone is done with the other slot
        if (step + 1 < n_steps) {
            const int nh2 = (step + 1) / tiles_per_head, nqt = qbeg + ((step + 1) % tiles_per_head) * BT2;
            copy_tile(smem + (slot ^ 1) * SLOT, g * group + nh2, nqt);
        }
        (void)hh;
        auto block = [&](auto B_) {
            constexpr int b = decltype(B_)::value;
            const int qb = qt + 32 * b;
            if (!((qb < w_hi_max) && (qb + 32 > w_lo_min))) return;
            // S[q, key] and dP[q, key]: rows = queries (registers), columns = keys (lanes); as assembly, so that the
            // results land in vector registers (see mfma_v), with the wait the vector ALU needs before it reads them
            f32x16 s, dp;
            static_for<0, KS>([&](auto K_) {
                constexpr int ks = decltype(K_)::value;
                const bf16x8 fq = frag_k<D>(sQ, 32 * b + l32, ks, half), fo = frag_k<D>(sdO, 32 * b + l32, ks, half);
                if constexpr (ks == 0) { mfma_v_first(s, fq, kf[0]); mfma_v_first(dp, fo, vf[0]); }
                else { mfma_v(s, fq, kf[ks]); mfma_v(dp, fo, vf[ks]); }
            });
            mfma_results_settle();
            const uint32_t tq = slot * SLOT, tdo = tq + TILE;
            // dO^T and Q^T fragments of MFMA 0 of the block
            shortx4 o0[4], o1[4], q0f[4], q1f[4];
            auto read_m = [&](auto M_) {
                constexpr int m = decltype(M_)::value;
                o0[0] = tr.template read<b, m, 0, 0>(tdo); o1[0] = tr.template read<b, m, 0, 1>(tdo);
                q0f[0] = tr.template read<b, m, 0, 0>(tq); q1f[0] = tr.template read<b, m, 0, 1>(tq);
                o0[1] = tr.template read<b, m, 1, 0>(tdo); o1[1] = tr.template read<b, m, 1, 1>(tdo);
                q0f[1] = tr.template read<b, m, 1, 0>(tq); q1f[1] = tr.template read<b, m, 1, 1>(tq);
                if (CB > 2) {
                    o0[2] = tr.template read<b, m, 2, 0>(tdo); o1[2] = tr.template read<b, m, 2, 1>(tdo);
                    q0f[2] = tr.template read<b, m, 2, 0>(tq); q1f[2] = tr.template read<b, m, 2, 1>(tq);
                    o0[3] = tr.template read<b, m, 3, 0>(tdo); o1[3] = tr.template read<b, m, 3, 1>(tdo);
                    q0f[3] = tr.template read<b, m, 3, 0>(tq); q1f[3] = tr.template read<b, m, 3, 1>(tq);
                } else {
                    o0[2] = o0[3] = o1[2] = o1[3] = q0f[2] = q0f[3] = q1f[2] = q1f[3] = shortx4{0, 0, 0, 0};
                }
            };
            read_m(std::integral_constant<int, 0>{});
            const bool inside = qb >= w_lo_max && qb + 32 <= w_hi_min;
            const unsigned span = (unsigned)(me.hi - me.lo);
            float p[16], ds[16];
            // two copies of the loop, so that a block no key of which is masked pays nothing for the mask
            auto softmax = [&](auto MASK_) {
                constexpr bool MASK = decltype(MASK_)::value;
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int r0 = 32 * b + 8 * gq + 4 * half;        // 4 consecutive queries
                    const float4 l4 = *reinterpret_cast<const float4 *>(sLse + r0);
                    const float4 d4 = *reinterpret_cast<const float4 *>(sD + r0);
                    const float lv[4] = {l4.x, l4.y, l4.z, l4.w}, dvv[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int i = 4 * gq + e;
                        float pv = __builtin_amdgcn_exp2f(fmaf(s[i], sl2, -lv[e] * LOG2E));
                        if (MASK) pv = (unsigned)(qt + r0 + e - me.lo) < span ? pv : 0.f;
                        p[i] = pv;
                        ds[i] = pv * (dp[i] + dvv[e]);                 // the D array holds -D
                    }
                }
            };
            if (inside) softmax(std::false_type{});
            else softmax(std::true_type{});
            asm volatile("s_waitcnt lgkmcnt(0)" : TR_WAIT4(o0), TR_WAIT4(o1), TR_WAIT4(q0f), TR_WAIT4(q1f));
            bf16x8 fo[4], fq[4];
#pragma unroll
            for (int c = 0; c < 4; ++c) { fo[c] = join(o0[c], o1[c]); fq[c] = join(q0f[c], q1f[c]); }
            read_m(std::integral_constant<int, 1>{});                 // in flight during the next 2 CB MFMAs
            {
                const bf16x8 pf = pack8(p), dsf = pack8(ds);
#pragma unroll
                for (int c = 0; c < CB; ++c) {
                    dv[c] = MFMA(fo[c], pf, dv[c]);
                    dk[c] = MFMA(fq[c], dsf, dk[c]);
                }
            }
            asm volatile("s_waitcnt lgkmcnt(0)" : TR_WAIT4(o0), TR_WAIT4(o1), TR_WAIT4(q0f), TR_WAIT4(q1f));
            {
                const bf16x8 pf = pack8(p + 8), dsf = pack8(ds + 8);
#pragma unroll
                for (int c = 0; c < CB; ++c) {
                    dv[c] = MFMA(join(o0[c], o1[c]), pf, dv[c]);
                    dk[c] = MFMA(join(q0f[c], q1f[c]), dsf, dk[c]);
                }
            }
        };
        block(std::integral_constant<int, 0>{});
        block(std::integral_constant<int, 1>{});
    }
    }
done:
    lds_barrier();                                     // the tiles are done with: LDS now stages the output rows
    {
        bf16_t *okp = (bf16_t *)a.d_qkv + (long)(k0 + wave * 32) * ld + nq + g * dh;
        uint8_t *stage = smem + wave * STAGE_BYTES<D>;
        store_rows<D, CB>(stage, dv, 1.f, okp + nk, ld, T - (k0 + wave * 32), dh);
        if (valid && a.rope_cs) unrotate<CB>(dk, a.rope_cs + (long)key * (D / 2), half);
        store_rows<D, CB>(stage, dk, a.scale, okp, ld, T - (k0 + wave * 32), dh);
    }
    add_busy(a.cu_busy ? a.cu_busy + 2048 : nullptr, true);
}

template <typename K>
hipError_t set_smem(K kern, int bytes) {
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
}

// Wavefronts per workgroup of the forward kernel: four for 64-wide heads (packs of ViT-sized segments: 0.068 -> 0.054 ms
// on the encoder workload), eight for 128-wide heads (no difference there within 2 %, and half the K / V tile traffic).
// The dQ kernel, which has the same structure, gains nothing from four (0.182 -> 0.185 ms backward on that workload).
template <int D>
constexpr int FWD_WAVES = D <= 64 ? 4 : 8;

template <int D>
hipError_t launch_fwd(const AttnArgs &a, hipStream_t st) {
    static std::atomic<bool> configured{false};     // set once; concurrent first calls repeat the same idempotent set-up
    constexpr int W = FWD_WAVES<D>;
    const int smem = std::max(2 * 2 * BT2 * D * 2 + (W == 4 ? 0 : W * ROWS32_BYTES<D>), W * STAGE_BYTES<D>);
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = set_smem(attn_fwd_kernel<D, W>, smem);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    attn_fwd_kernel<D, W><<<dim3(a.nh, ceil_div(a.T, FQ) * (FQ / (W * 32))), W * 64, smem, st>>>(a);
    return hipGetLastError();
}

template <int D>
hipError_t launch_bwd(const AttnArgs &a, hipStream_t st) {
    static std::atomic<bool> configured{false};     // set once; concurrent first calls repeat the same idempotent set-up
    constexpr bool PIPELINED = D > 64;                  // see attn_dkv_plain_kernel
    constexpr int DKV_SLOT = 2 * BT2 * D * 2 + 2 * BT2 * 4;
    const int smem_dq = std::max(DQ_LDS_BYTES<D>, 8 * STAGE_BYTES<D>), smem_dkv = PIPELINED ? 3 * DKV_SLOT + DKV_STAGE_BYTES<D> : 2 * DKV_SLOT + 2 * DKV_STAGE_BYTES<D>;
    if (!configured.load(std::memory_order_acquire)) {
        hipError_t e = set_smem(attn_dq_kernel<D>, smem_dq);
        if (e != hipSuccess) return e;
        if constexpr (PIPELINED) e = set_smem(attn_dkv_kernel<D>, smem_dkv);
        else e = set_smem(attn_dkv_plain_kernel<D>, smem_dkv);
        if (e != hipSuccess) return e;
        configured.store(true, std::memory_order_release);
    }
    attn_dq_kernel<D><<<dim3(a.nh, ceil_div(a.T, FQ)), 512, smem_dq, st>>>(a);
    if constexpr (PIPELINED) attn_dkv_kernel<D><<<dim3(a.nkv, ceil_div(a.T, BQ)), 256, smem_dkv, st>>>(a);
    else attn_dkv_plain_kernel<D><<<dim3(a.nkv, ceil_div(a.T, BQ)), 256, smem_dkv, st>>>(a);
    return hipGetLastError();
}

}  // namespace

hipError_t attn_mfma_fwd(const AttnArgs &a, hipStream_t st) {
    if (a.T == 0) return hipSuccess;
    if ((size_t)a.T * a.ld_qkv * 2 >= MAX_TENSOR_BYTES) return hipErrorInvalidValue;
    return a.d <= 64 ? launch_fwd<64>(a, st) : launch_fwd<128>(a, st);
}

hipError_t attn_mfma_bwd(const AttnArgs &a, hipStream_t st) {
    if (a.T == 0) return hipSuccess;
    if ((size_t)a.T * a.ld_qkv * 2 >= MAX_TENSOR_BYTES) return hipErrorInvalidValue;
    return a.d <= 64 ? launch_bwd<64>(a, st) : launch_bwd<128>(a, st);
}

}  // namespace mmt
