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
void attn_tile_order(const int32_t *cu, const uint8_t *modes, int default_mode, int S, int T, AttnArgs &a) {
    constexpr int FQ = 256, BK = 128;
    const int nq = (T + FQ - 1) / FQ, nk = (T + BK - 1) / BK;
    a.use_order = 0;
    if (nq > (int)sizeof(a.order_q) || nk > (int)sizeof(a.order_k) || T == 0) return;
    std::vector<int> seg_of(T);
    for (int s = 0; s < S; ++s)
        for (int t = cu[s]; t < cu[s + 1]; ++t) seg_of[t] = s;
    auto bidir = [&](int s) { return (modes ? modes[s] : default_mode) == MASK_BIDIR; };
    std::vector<double> wq(nq), wk(nk);
    for (int i = 0; i < nq; ++i) {
        const int q0 = i * FQ, q1 = std::min(q0 + FQ, T) - 1;
        const int lo = cu[seg_of[q0]], hi = bidir(seg_of[q1]) ? cu[seg_of[q1] + 1] : q1 + 1;
        wq[i] = (hi - lo + 63) / 64;
    }
    for (int i = 0; i < nk; ++i) {
        const int k0 = i * BK, k1 = std::min(k0 + BK, T) - 1;
        const int lo = bidir(seg_of[k0]) ? cu[seg_of[k0]] : k0, hi = cu[seg_of[k1] + 1];
        wk[i] = (hi - lo + 63) / 64;
    }
    std::vector<int> idx;
    sort_desc(wq.data(), nq, idx);
    for (int i = 0; i < nq; ++i) a.order_q[i] = (uint8_t)idx[i];
    sort_desc(wk.data(), nk, idx);
    for (int i = 0; i < nk; ++i) a.order_k[i] = (uint8_t)idx[i];
    a.use_order = 1;
}

}  // namespace mmt
