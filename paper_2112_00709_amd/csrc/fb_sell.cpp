// Host-side construction of the sliced plans the recursion kernel walks.
//
// The forward recursion (Eq. 13) multiplies by T transposed: row j of the
// product gathers the arcs that enter state j.  The backward recursion (Eq. 14)
// multiplies by T: row i gathers the arcs that leave state i.  Both are sparse
// matrix x vector products in the log semifield.  This file turns such a matrix
// into a static work plan for one workgroup:
//   * 64 lanes per slice; a row of up to kChunk arcs takes one lane, a longer one 2, 4, ... 64
//     lanes of one slice so that no lane walks more than kChunkWide arcs, and all rows of a
//     slice take the same number of lanes (the kernel adds the lanes of a row up when the slice ends);
//   * a row too long even for 64 lanes is cloned: the clones are rows of their own
//     whose values the next step gathers like any other state (the arcs that leave
//     the row's state are repeated for every clone), so in-degree skew costs
//     neither a second pass nor a workgroup barrier;
//   * rows sorted by length so that a slice is padded little; rows without arcs
//     are left out (their value is the semiring zero at every step but the first);
//   * slices of rows with one or two arcs are stacked four (two) to a batch;
//   * slices are dealt to the waves of the workgroup longest-first, so every
//     wave walks about the same number of batches per time step.
#include <algorithm>
#include <cmath>
#include <numeric>
#include <utility>

#include "fb_internal.h"

namespace fb {

namespace {

struct Item {
    int32_t out;       // target: state, or K + clone slot
    int32_t vidx;
    int64_t begin;     // range in the expanded arc pool
    int32_t n;
};

int lanes_log2(int32_t n)
{
    int lg = 0;
    while (lg < 6 && (n + (1 << lg) - 1) / (1 << lg) > (lg == 0 ? kChunk : kChunkWide)) ++lg;
    return lg;
}

// batches of the stream a slice of this width takes
int32_t slice_batches(int32_t trip) { return (trip + kBatchRows - 1) / kBatchRows; }

}  // namespace

void sell_append(SellHost &S, int32_t k0, int32_t K, const int64_t *ptr, const int32_t *col, const float *w,
                 const int32_t *row_vidx)
{
    const int nw = S.nw;
    SubDesc sd{};
    sd.k0 = k0;
    sd.K = K;
    sd.wave_ptr0 = (int32_t)S.wave_ptr.size();
    sd.clone0 = (int32_t)S.clones.size();
    sd.zero0 = (int32_t)S.zero_rows.size();

    // rows that need clones, and their slots
    const int64_t row_cap = (int64_t)kWave * kChunkWide;
    std::vector<int32_t> n_share((size_t)K, 1), first_slot((size_t)K, 0);
    int32_t n_slot = 0;
    for (int32_t r = 0; r < K; ++r) {
        const int64_t n = ptr[r + 1] - ptr[r];
        if (n <= row_cap) continue;
        n_share[r] = (int32_t)((n + row_cap - 1) / row_cap);
        first_slot[r] = n_slot;
        S.clones.push_back(CloneDesc{r, n_slot, n_share[r] - 1, 0});
        n_slot += n_share[r] - 1;
    }
    sd.n_slot = n_slot;
    sd.n_cdesc = (int32_t)S.clones.size() - sd.clone0;

    // arc pool with the arcs out of cloned states repeated, then one item per row or clone
    std::vector<int32_t> pcol;
    std::vector<float> pw;
    std::vector<Item> items;
    for (int32_t r = 0; r < K; ++r) {
        const int64_t begin = (int64_t)pcol.size();
        for (int64_t e = ptr[r]; e < ptr[r + 1]; ++e) {
            pcol.push_back(col[e]);
            pw.push_back(w[e]);
            for (int32_t c = 1; c < n_share[col[e]]; ++c) {
                pcol.push_back(K + first_slot[col[e]] + c - 1);
                pw.push_back(w[e]);
            }
        }
        const int64_t n = (int64_t)pcol.size() - begin;
        if (n == 0) {
            S.zero_rows.push_back(r);
            continue;
        }
        const int32_t shares = n_share[r];
        int64_t at = begin;
        for (int32_t c = 0; c < shares; ++c) {
            const int32_t len = (int32_t)(n / shares + (c < n % shares ? 1 : 0));
            items.push_back(Item{c == 0 ? r : K + first_slot[r] + c - 1, row_vidx[r], at, len});
            at += len;
        }
    }
    sd.n_zero = (int32_t)S.zero_rows.size() - sd.zero0;

    // longest rows first (stable: equal lengths keep row order); a slice takes its lanes-per-row from
    // its first (longest) row, the rows after it are not longer and fit the same share of lanes
    std::stable_sort(items.begin(), items.end(), [](const Item &a, const Item &b) { return a.n > b.n; });
    struct Slice { size_t first; int32_t count, lg, trip; };
    std::vector<Slice> slices;
    for (size_t i = 0; i < items.size();) {
        Slice sl{};
        sl.first = i;
        sl.lg = lanes_log2(items[i].n);
        sl.count = (int32_t)std::min<size_t>((size_t)(kWave >> sl.lg), items.size() - i);
        sl.trip = (items[i].n + (1 << sl.lg) - 1) >> sl.lg;
        slices.push_back(sl);
        i += (size_t)sl.count;
    }
    // Slices whose rows have one arc (or at most two) are stacked, four (two) of them to a batch: a lane then
    // works on four (two) rows of different slices at once and no batch is three quarters (half) padding.
    // Stacked batches have a kernel path of their own that exists only for the first batches of a wave's step,
    // so a wave takes at most kMaxStacked of them and they come first in its list.
    struct Unit { int stack; size_t sub[kBatchRows]; int n_sub; int64_t batches; };
    std::vector<Unit> stacked, plain;
    {
        std::vector<size_t> one, two;
        for (size_t s = 0; s < slices.size(); ++s) {
            if (slices[s].lg == 0 && slices[s].trip == 1) one.push_back(s);
            else if (slices[s].lg == 0 && slices[s].trip == 2) two.push_back(s);
            else plain.push_back(Unit{0, {s, 0, 0, 0}, 1, slice_batches(slices[s].trip)});
        }
        auto group = [&](const std::vector<size_t> &v, int stack) {
            for (size_t i = 0; i < v.size(); i += (size_t)stack) {
                Unit u{stack, {0, 0, 0, 0}, 0, 1};
                for (size_t j = i; j < v.size() && j < i + (size_t)stack; ++j) u.sub[u.n_sub++] = v[j];
                if (u.n_sub == 1) plain.push_back(Unit{0, {u.sub[0], 0, 0, 0}, 1, 1});   // nothing to stack it with
                else stacked.push_back(u);
            }
        };
        group(two, 2);
        group(one, kBatchRows);
    }
    // deal to waves: most batches first, to the wave that would finish first
    // Waves go round the four SIMDs of a compute unit.  In a 16-wave workgroup the last SIMD hosts the
    // data-moving wave in place of a fourth arc-walking one, so its three arc-walking waves run a little
    // faster than the others and take a little more (measured: a tenth more is best).
    std::vector<std::vector<Unit>> mine((size_t)nw);
    std::vector<int64_t> load((size_t)nw, 0);
    std::vector<int> n_stacked((size_t)nw, 0);
    auto finish = [&](int wv, int64_t nbat) {
        return (double)(load[wv] + nbat) / ((nw == kNWShared - 1 && wv % 4 == 3) ? 1.1 : 1.0);
    };
    for (const Unit &u : stacked) {
        int best = -1;
        for (int wv = 0; wv < nw; ++wv)
            if (n_stacked[wv] < kMaxStacked && (best < 0 || finish(wv, 1) < finish(best, 1))) best = wv;
        if (best < 0) {   // every wave has its fill of stacked batches: these slices stay plain
            for (int j = 0; j < u.n_sub; ++j) plain.push_back(Unit{0, {u.sub[j], 0, 0, 0}, 1, 1});
            continue;
        }
        mine[best].push_back(u);
        load[best] += 1;
        ++n_stacked[best];
    }
    std::stable_sort(plain.begin(), plain.end(), [&](const Unit &a, const Unit &b) { return a.batches > b.batches; });
    for (const Unit &u : plain) {
        int best = 0;
        for (int wv = 1; wv < nw; ++wv)
            if (finish(wv, u.batches) < finish(best, u.batches)) best = wv;
        mine[best].push_back(u);
        load[best] += u.batches;
    }
    for (int wv = 0; wv < nw; ++wv) {
        S.wave_ptr.push_back((int32_t)S.slice_trip.size());
        for (const Unit &u : mine[wv]) {
            if (u.stack) {
                // one batch: part t of a lane = the lane's row of slice u.sub[t], kBatchRows / stack rows each
                const int rows_per = kBatchRows / u.stack;
                S.slice_trip.push_back(kBatchRows);
                S.slice_lg.push_back(0);
                S.slice_stack.push_back(u.stack);
                S.slice_arc.push_back((int64_t)S.arcs.size());
                for (int lane = 0; lane < kWave; ++lane)
                    for (int part = 0; part < kBatchRows; ++part) {
                        const bool live = part < u.n_sub && lane < slices[u.sub[part]].count;
                        S.row_out.push_back(live ? items[slices[u.sub[part]].first + (size_t)lane].out : -1);
                        S.row_vidx.push_back(live ? items[slices[u.sub[part]].first + (size_t)lane].vidx : -1);
                    }
                for (int row = 0; row < kBatchRows; ++row)
                    for (int lane = 0; lane < kWave; ++lane) {
                        Arc a{0, -INFINITY};
                        const int part = row / rows_per, j = row % rows_per;
                        if (part < u.n_sub && lane < slices[u.sub[part]].count) {
                            const Item &im = items[slices[u.sub[part]].first + (size_t)lane];
                            if (j < im.n) {
                                a.src = pcol[(size_t)(im.begin + j)];
                                a.w = pw[(size_t)(im.begin + j)];
                            }
                        }
                        S.arcs.push_back(a);
                    }
                continue;
            }
            const Slice &sl = slices[u.sub[0]];
            const int g = 1 << sl.lg;
            S.slice_trip.push_back(sl.trip);
            S.slice_lg.push_back(sl.lg);
            S.slice_stack.push_back(0);
            S.slice_arc.push_back((int64_t)S.arcs.size());
            for (int lane = 0; lane < kWave; ++lane) {
                const int it = lane >> sl.lg;
                const bool live = it < sl.count;
                for (int part = 0; part < kBatchRows; ++part) {
                    S.row_out.push_back(part == 0 && live && (lane & (g - 1)) == 0 ? items[sl.first + it].out : -1);
                    S.row_vidx.push_back(part == 0 && live ? items[sl.first + it].vidx : -1);
                }
            }
            // lane t of a row's g lanes walks arcs [t * trip, (t + 1) * trip) of the row
            for (int32_t step = 0; step < sl.trip; ++step)
                for (int lane = 0; lane < kWave; ++lane) {
                    Arc a{0, -INFINITY};
                    const int it = lane >> sl.lg;
                    if (it < sl.count) {
                        const Item &im = items[sl.first + it];
                        const int64_t j = (int64_t)(lane & (g - 1)) * sl.trip + step;
                        if (j < im.n) {
                            a.src = pcol[(size_t)(im.begin + j)];
                            a.w = pw[(size_t)(im.begin + j)];
                        }
                    }
                    S.arcs.push_back(a);
                }
        }
    }
    S.wave_ptr.push_back((int32_t)S.slice_trip.size());   // end of the last wave's range
    S.max_slot = std::max(S.max_slot, n_slot);
    S.sub.push_back(sd);
}

// Every index a kernel will dereference while walking the plan stays inside the arrays it
// indexes.  n_vidx: entries of the staged emission vector; a negative value means "the
// sub-graph's own state count".
bool sell_in_bounds(const SellHost &S, int32_t n_vidx, std::string &why)
{
    const size_t n_slices = S.slice_trip.size();
    if (S.slice_arc.size() != n_slices || S.slice_lg.size() != n_slices || S.slice_stack.size() != n_slices ||
        S.row_out.size() != n_slices * kWave * kBatchRows || S.row_vidx.size() != n_slices * kWave * kBatchRows) {
        why = "slice arrays disagree in size";
        return false;
    }
    for (const SubDesc &sd : S.sub) {
        if (sd.wave_ptr0 < 0 || (size_t)sd.wave_ptr0 + (size_t)S.nw + 1 > S.wave_ptr.size()) { why = "wave_ptr range"; return false; }
        if (sd.clone0 < 0 || sd.n_cdesc < 0 || (size_t)sd.clone0 + (size_t)sd.n_cdesc > S.clones.size()) { why = "clone range"; return false; }
        if (sd.zero0 < 0 || sd.n_zero < 0 || (size_t)sd.zero0 + (size_t)sd.n_zero > S.zero_rows.size()) { why = "zero-row range"; return false; }
        for (int32_t c = 0; c < sd.n_cdesc; ++c) {
            const CloneDesc &cd = S.clones[(size_t)sd.clone0 + c];
            if (cd.state < 0 || cd.state >= sd.K || cd.first < 0 || cd.count < 1 || cd.first + cd.count > sd.n_slot) { why = "clone entry"; return false; }
        }
        for (int32_t z = 0; z < sd.n_zero; ++z)
            if (S.zero_rows[(size_t)sd.zero0 + z] < 0 || S.zero_rows[(size_t)sd.zero0 + z] >= sd.K) { why = "zero row"; return false; }
        const int32_t n_idx = sd.K + sd.n_slot;
        for (int wv = 0; wv < S.nw; ++wv) {
            const int32_t s0 = S.wave_ptr[(size_t)sd.wave_ptr0 + wv], s1 = S.wave_ptr[(size_t)sd.wave_ptr0 + wv + 1];
            if (s0 < 0 || s1 < s0 || (size_t)s1 > n_slices) { why = "slice range"; return false; }
            int n_stacked = 0;
            for (int32_t s = s0; s < s1; ++s) {
                const int32_t trip = S.slice_trip[s], stack = S.slice_stack[s];
                if (trip < 1) { why = "trip count"; return false; }
                if (S.slice_lg[s] < 0 || S.slice_lg[s] > 6) { why = "lanes per row"; return false; }
                if (stack != 0 && stack != 2 && stack != kBatchRows) { why = "stack size"; return false; }
                if (stack && (trip != kBatchRows || S.slice_lg[s] != 0 || s - s0 != n_stacked || ++n_stacked > kMaxStacked)) {
                    why = "stacked slice";   // one batch, one lane per row, first in the wave's list, at most kMaxStacked
                    return false;
                }
                if (S.slice_arc[s] < 0 || (size_t)S.slice_arc[s] + (size_t)trip * kWave > S.arcs.size()) { why = "arc range"; return false; }
                for (size_t a = (size_t)S.slice_arc[s]; a < (size_t)S.slice_arc[s] + (size_t)trip * kWave; ++a)
                    if (S.arcs[a].src < 0 || S.arcs[a].src >= n_idx) { why = "arc source"; return false; }
                for (int e = 0; e < kWave * kBatchRows; ++e) {
                    const int32_t o = S.row_out[(size_t)s * kWave * kBatchRows + e], v = S.row_vidx[(size_t)s * kWave * kBatchRows + e];
                    if (o < -1 || o >= n_idx) { why = "row target"; return false; }
                    if (v < -1 || v >= std::max(n_vidx < 0 ? sd.K : n_vidx, 1)) { why = "emission index"; return false; }
                    if (o >= 0 && v < 0) { why = "row without emission index"; return false; }
                    if (o >= 0 && e % kBatchRows >= std::max(stack, 1)) { why = "target of a part the slice does not have"; return false; }
                }
            }
        }
    }
    return true;
}

}  // namespace fb
