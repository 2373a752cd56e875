// Longest-first greedy partitioning (Algorithm 1, intra-microbatch reordering): host code only.
//
// The n samples are sorted by size in descending order and handed out one by one, each to the group whose
// load is currently the smallest; the result is the concatenation of the groups.  Two choices the
// algorithm leaves open are fixed by the paper's worked example (four samples of which the first two are
// the largest, two groups, result order 1 3 2 4): equal sizes keep their original order (stable sort),
// and among equally loaded groups the one with the lowest index is taken.
//
// The same ordering is used inside the GPU for the attention kernels' work items (tile_order below): tiles
// are dispatched heaviest first, so that the short ones fill the gaps at the end of the launch.
#include "kernels.h"
#include <algorithm>
#include <numeric>
#include <vector>

namespace mmt {

// indices 0..n-1 sorted by cost, descending, ties in index order
static void sort_desc(const double *cost, int n, std::vector<int> &idx) {
    idx.resize(n);
    std::iota(idx.begin(), idx.end(), 0);
    std::stable_sort(idx.begin(), idx.end(), [&](int a, int b) { return cost[a] > cost[b]; });
}

int intra_reorder(const double *sizes, int n, int m, int32_t *order, int32_t *group_begin, double *group_load) {
    std::vector<int> sorted;
    sort_desc(sizes, n, sorted);
    std::vector<std::vector<int>> groups(m);
    std::vector<double> load(m, 0.0);
    for (int i = 0; i < n; ++i) {
        int best = 0;
        for (int j = 1; j < m; ++j)
            if (load[j] < load[best]) best = j;           // strict: ties stay with the lowest index
        groups[best].push_back(sorted[i]);
        load[best] += sizes[sorted[i]];
    }
    int pos = 0;
    for (int j = 0; j < m; ++j) {
        if (group_begin) group_begin[j] = pos;
        for (int s : groups[j]) order[pos++] = s;
        if (group_load) group_load[j] = load[j];
    }
    if (group_begin) group_begin[m] = pos;
    return 0;
}

// Work of the attention kernels' tiles, from the host copy of the segment offsets:
//   query tile (FQ queries): 64-key steps between the first query's segment start and the last query's last key;
//   key tile (BQ keys): 64-query steps between the first key's first query and the last key's segment end.
// Runs on the launch path of every attention call, so it allocates nothing: the segments of the tiles' first and
// last tokens come from one walk over the offsets (tile starts increase), the two tables are sorted in place, and
// the result of the last pack is kept per thread -- forward, backward and every layer of a stack pass the same
// pack, which is recognised by a hash of its offsets and mask modes.
namespace {
struct TileOrderCache {
    uint64_t key = 0;
    int S = -1, T = -1, default_mode = -1, use_order = 0;
    uint8_t order_q[sizeof(AttnArgs::order_q)], order_k[sizeof(AttnArgs::order_k)];
};
thread_local TileOrderCache g_tile_order;

uint64_t pack_hash(const int32_t *cu, const uint8_t *modes, int S) {
    uint64_t h = 1469598103934665603ull;                       // FNV-1a over the offsets, then the modes
    auto mix = [&](uint64_t v) { h = (h ^ v) * 1099511628211ull; };
    for (int s = 0; s <= S; ++s) mix((uint32_t)cu[s]);
    mix(modes ? 0x100 : 0x200);
    if (modes) for (int s = 0; s < S; ++s) mix(modes[s]);
    return h;
}

// idx[0..n) = 0..n-1 sorted by weight, descending, equal weights in index order (insertion sort: n <= 128)
void order_desc(const int *w, int n, uint8_t *idx) {
    for (int i = 0; i < n; ++i) {
        int j = i;
        while (j > 0 && w[idx[j - 1]] < w[i]) { idx[j] = idx[j - 1]; --j; }
        idx[j] = (uint8_t)i;
    }
}
}  // namespace

void attn_tile_order(const int32_t *cu, const uint8_t *modes, int default_mode, int S, int T, AttnArgs &a) {
    constexpr int FQ = 256, BK = 128, MAXQ = (int)sizeof(a.order_q), MAXK = (int)sizeof(a.order_k);
    const int nq = (T + FQ - 1) / FQ, nk = (T + BK - 1) / BK;
    a.use_order = 0;
    if (nq > MAXQ || nk > MAXK || T == 0) return;              // more tiles than the tables hold: index order
    TileOrderCache &c = g_tile_order;
    const uint64_t key = pack_hash(cu, modes, S);
    if (!(c.key == key && c.S == S && c.T == T && c.default_mode == default_mode)) {
        auto bidir = [&](int s) { return (modes ? modes[s] : default_mode) == MASK_BIDIR; };
        int wq[MAXQ], wk[MAXK];
        int s = 0;                                             // segment of token t: the tokens asked for only increase
        auto seg_of = [&](int t) { while (cu[s + 1] <= t) ++s; return s; };
        for (int i = 0; i < nq; ++i) {
            const int q0 = i * FQ, q1 = std::min(q0 + FQ, T) - 1;
            const int lo = cu[seg_of(q0)], s1 = seg_of(q1), hi = bidir(s1) ? cu[s1 + 1] : q1 + 1;
            wq[i] = (hi - lo + 63) / 64;
        }
        s = 0;
        for (int i = 0; i < nk; ++i) {
            const int k0 = i * BK, k1 = std::min(k0 + BK, T) - 1;
            const int s0 = seg_of(k0), lo = bidir(s0) ? cu[s0] : k0, hi = cu[seg_of(k1) + 1];
            wk[i] = (hi - lo + 63) / 64;
        }
        order_desc(wq, nq, c.order_q);
        order_desc(wk, nk, c.order_k);
        c.key = key; c.S = S; c.T = T; c.default_mode = default_mode; c.use_order = 1;
    }
    for (int i = 0; i < nq; ++i) a.order_q[i] = c.order_q[i];
    for (int i = 0; i < nk; ++i) a.order_k[i] = c.order_k[i];
    a.use_order = 1;
}

}  // namespace mmt
