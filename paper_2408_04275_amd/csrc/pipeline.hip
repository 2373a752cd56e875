// One-forward-one-backward pipeline timeline and inter-microbatch reordering (Algorithm 2, Section
// "Inter-microbatch Reordering"): host code only.
//
// Timeline.  Stage s of p runs min(p - 1 - s, l) warm-up forward passes, then forward / backward pairs, then the
// backward passes that are left.  An operation starts when the previous operation of its stage and the producer of
// its input (the same microbatch's forward pass one stage up, or its backward pass one stage down) have both ended.
// The timeline is evaluated by a sweep that keeps one cursor per stage and moves a cursor as long as the next
// operation's input exists; every operation is evaluated once.
//
// Reordering.  The smallest microbatch goes first, the p - 1 smallest of the rest go last, and the positions in
// between are filled interval by interval: interval i at the first stage is the wait for backward pass i (after the
// first forward pass for i = 1, after backward pass i - 1 otherwise), filled by the forward passes 2 .. p (i = 1) or by
// forward pass i + p - 1, and the microbatches whose first-stage forward time comes closest to the interval are put
// there.  The same sweep serves as GETINTERVAL: cursors stop in front of a position that is still empty, so placing a
// microbatch costs O(p) further operations, and interval i never depends on an empty position (interval 1 aside,
// which is the first microbatch's way through stages 2 .. p and back).
// A microbatch's size (MIN, SELECTMIN) is, as the section defines it, its computation time in the modality encoder
// and the generator, the modules whose time varies with the data: the caller passes it per microbatch, or, without
// one, it is taken as the forward + backward time of the first and the last stage (the encoder's and the generator's
// stage of a three-module pipeline).
// Choices the listing leaves open: equal sizes and equal
// distances go to the lowest index; the rear is in ascending order of size; the loop runs while microbatches remain
// (the listing's l - p iterations would hand out more microbatches than there are); when k microbatches are picked
// for one interval, each pick aims at the volume still open divided by the picks still to make.
#include "kernels.h"
#include <algorithm>
#include <cmath>
#include <vector>

namespace mmt {

namespace {

struct Timeline {
    int p, l;
    const double *fwd, *bwd;            // [p][l], indexed by original microbatch
    std::vector<int> at;                // microbatch at each position; -1: empty
    std::vector<double> endF, endB;     // [p][l] by position
    std::vector<char> haveF, haveB;
    std::vector<int> cursor;            // per stage: operations evaluated so far
    std::vector<double> free_at;        // per stage: end of the last evaluated operation

    Timeline(int p_, int l_, const double *f, const double *b)
        : p(p_), l(l_), fwd(f), bwd(b), at(l_, -1), endF((size_t)p_ * l_, 0.0), endB((size_t)p_ * l_, 0.0),
          haveF((size_t)p_ * l_, 0), haveB((size_t)p_ * l_, 0), cursor(p_, 0), free_at(p_, 0.0) {}

    // operation number c of stage s: is it a forward pass, and of which position
    void op_at(int s, int c, bool &is_f, int &pos) const {
        const int warm = std::min(p - 1 - s, l);
        if (c < warm) { is_f = true; pos = c; return; }
        const int pairs = l - warm, r = c - warm;
        if (r < 2 * pairs) { is_f = !(r & 1); pos = is_f ? warm + r / 2 : r / 2; return; }
        is_f = false; pos = pairs + (r - 2 * pairs);
    }
    // moves every stage's cursor as far as inputs and filled positions allow
    void sweep() {
        bool moved = true;
        while (moved) {
            moved = false;
            for (int s = 0; s < p; ++s) {
                while (cursor[s] < 2 * l) {
                    bool is_f; int pos;
                    op_at(s, cursor[s], is_f, pos);
                    if (at[pos] < 0) break;
                    const size_t me = (size_t)s * l + pos;
                    double input = 0.0;
                    if (is_f) {
                        if (s > 0) { if (!haveF[me - l]) break; input = endF[me - l]; }
                    } else if (s < p - 1) { if (!haveB[me + l]) break; input = endB[me + l]; }
                    else { if (!haveF[me]) break; input = endF[me]; }
                    const double dur = (is_f ? fwd : bwd)[(size_t)s * l + at[pos]];
                    const double t = std::max(free_at[s], input) + dur;
                    if (is_f) { endF[me] = t; haveF[me] = 1; } else { endB[me] = t; haveB[me] = 1; }
                    free_at[s] = t;
                    ++cursor[s];
                    moved = true;
                }
            }
        }
    }
    // interval i (1-based) at the first stage; every operation it refers to has been evaluated
    double interval(int i) const {
        if (p == 1) return 0.0;
        const double anchor = i == 1 ? endF[0] : endB[i - 2];
        const double ready = endB[(size_t)l + i - 1];
        return std::max(0.0, ready - anchor);
    }
};

}  // namespace

int pipeline_1f1b(const double *fwd, const double *bwd, int p, int l, const int32_t *order, double *makespan,
                  double *intervals) {
    Timeline tl(p, l, fwd, bwd);
    for (int q = 0; q < l; ++q) tl.at[q] = order ? order[q] : q;
    tl.sweep();
    double end = 0.0;
    for (int s = 0; s < p; ++s) {
        if (tl.cursor[s] != 2 * l) return 1;          // cannot happen for this schedule
        end = std::max(end, tl.free_at[s]);
    }
    if (makespan) *makespan = end;
    if (intervals)
        for (int i = 1; i <= l; ++i) {
            // with a single stage a backward pass waits for nothing but its own forward pass
            if (p == 1) intervals[i - 1] = std::max(0.0, tl.endF[i - 1] - (i == 1 ? tl.endF[0] : tl.endB[i - 2]));
            else intervals[i - 1] = tl.interval(i);
        }
    return 0;
}

int inter_reorder(const double *fwd, const double *bwd, int p, int l, const double *sizes, int32_t *order,
                  double *intervals_seen, int32_t *n_seen) {
    if (n_seen) *n_seen = 0;
    if (l == 0) return 0;
    std::vector<double> size(l, 0.0);
    for (int j = 0; j < l; ++j) {
        if (sizes) { size[j] = sizes[j]; continue; }
        size[j] = fwd[j] + bwd[j];                                                   // first stage: the modality encoder
        if (p > 1) size[j] += fwd[(size_t)(p - 1) * l + j] + bwd[(size_t)(p - 1) * l + j];   // last stage: the generator
    }
    std::vector<char> taken(l, 0);
    auto take_min = [&]() {
        int best = -1;
        for (int j = 0; j < l; ++j)
            if (!taken[j] && (best < 0 || size[j] < size[best])) best = j;
        taken[best] = 1;
        return best;
    };
    Timeline tl(p, l, fwd, bwd);
    int placed = 0, left = l;
    auto place = [&](int m) { tl.at[placed] = m; order[placed++] = m; };
    place(take_min()); --left;
    std::vector<int> rear;
    for (int r = 0; r < p - 1 && left > 0; ++r) { rear.push_back(take_min()); --left; }
    tl.sweep();
    const int first = order[0];
    for (int i = 1; left > 0; ++i) {
        double volume;
        if (i == 1) {                      // nothing but the first microbatch is in the pipeline yet
            volume = 0.0;
            for (int s = 1; s < p; ++s) volume += fwd[(size_t)s * l + first] + bwd[(size_t)s * l + first];
        } else volume = tl.interval(i);
        if (intervals_seen) intervals_seen[i - 1] = volume;
        if (n_seen) *n_seen = i;
        const int picks = std::min(i == 1 ? p - 1 : 1, left);
        for (int r = 0; r < picks; ++r) {
            const double target = volume / (picks - r);
            int best = -1;
            double best_dist = 0.0;
            for (int j = 0; j < l; ++j) {
                if (taken[j]) continue;
                const double dist = std::fabs(fwd[j] - target);
                if (best < 0 || dist < best_dist) { best = j; best_dist = dist; }
            }
            taken[best] = 1; --left;
            volume -= fwd[best];
            place(best);
        }
        tl.sweep();
    }
    for (int m : rear) place(m);
    return 0;
}

}  // namespace mmt
