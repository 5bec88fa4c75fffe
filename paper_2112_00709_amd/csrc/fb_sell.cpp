// Host-side construction of the row-split sliced-ELL schedules the kernels walk.
//
// The forward recursion (Eq. 13) multiplies by T transposed: row j of the
// product gathers the arcs that enter state j.  The backward recursion (Eq. 14)
// multiplies by T: row i gathers the arcs that leave state i.  Both are sparse
// matrix x vector products in the log semifield, and so is (in ordinary
// arithmetic) the accumulation of state posteriors into pdf posteriors.  This
// file turns any such matrix into a static work plan for one workgroup:
//   * one row per lane, 64 rows per slice, slice padded to its longest row;
//   * rows sorted by length so that padding is small;
//   * a row longer than kChunk entries is cut into partial rows; the partial
//     results land in numbered slots and the next level combines them with the
//     same row-per-lane loop (in-degree skew never leaves a lane alone with
//     thousands of arcs);
//   * slices are dealt to the waves of the workgroup longest-first, so every
//     wave walks about the same number of arcs between two barriers.
#include <algorithm>
#include <cmath>
#include <numeric>
#include <utility>

#include "fb_internal.h"

namespace fb {

namespace {

struct Item {
    int32_t out;       // row_out encoding
    int32_t vidx;
    int64_t begin;     // range in the level's entry pool
    int32_t n;
};

}  // namespace

void sell_append(SellHost &S, int32_t k0, int32_t K, int32_t n_rows, const int64_t *ptr, const int32_t *col,
                 const float *w, const int32_t *row_out_id, const int32_t *row_vidx_id, float pad_w, float one_w)
{
    const int nw = S.nw;
    SubDesc sd{};
    sd.k0 = k0;
    sd.K = K;
    sd.wave_ptr0 = (int32_t)S.wave_ptr.size();

    // entry pool of the current level
    std::vector<int32_t> pcol(col, col + ptr[n_rows]);
    std::vector<float> pw(w, w + ptr[n_rows]);
    struct Row { int32_t out, vidx; int64_t begin; int32_t n; };
    std::vector<Row> rows(n_rows);
    for (int32_t r = 0; r < n_rows; ++r)
        rows[r] = Row{row_out_id[r], row_vidx_id ? row_vidx_id[r] : 0, ptr[r], (int32_t)(ptr[r + 1] - ptr[r])};

    int32_t n_part = 0, n_levels = 0;
    while (!rows.empty()) {
        std::vector<Item> items;
        std::vector<Row> next_rows;
        std::vector<int32_t> ncol;
        std::vector<float> nwgt;
        for (const Row &r : rows) {
            if (r.n <= kChunk) {
                items.push_back(Item{r.out, r.vidx, r.begin, r.n});
                continue;
            }
            int32_t nch = (r.n + kChunk - 1) / kChunk, base = r.n / nch, rem = r.n % nch;
            int64_t at = r.begin;
            Row nr{r.out, r.vidx, (int64_t)ncol.size(), nch};
            for (int32_t c = 0; c < nch; ++c) {
                int32_t len = base + (c < rem ? 1 : 0);
                items.push_back(Item{-2 - n_part, 0, at, len});
                ncol.push_back(n_part);
                nwgt.push_back(one_w);
                ++n_part;
                at += len;
            }
            next_rows.push_back(nr);
        }
        // longest rows first (stable: equal lengths keep row order)
        std::stable_sort(items.begin(), items.end(), [](const Item &a, const Item &b) { return a.n > b.n; });
        const int32_t n_sl = (int32_t)((items.size() + kWave - 1) / kWave);
        // deal slices to waves: longest first, to the least loaded wave
        std::vector<std::vector<int32_t>> mine(nw);
        std::vector<int64_t> load(nw, 0);
        for (int32_t s = 0; s < n_sl; ++s) {
            int best = 0;
            for (int wv = 1; wv < nw; ++wv)
                if (load[wv] < load[best]) best = wv;
            mine[best].push_back(s);
            load[best] += items[(size_t)s * kWave].n + 3;   // +3: fixed cost of a slice in arc visits
        }
        for (int wv = 0; wv < nw; ++wv) {
            S.wave_ptr.push_back((int32_t)S.slice_trip.size());
            for (int32_t s : mine[wv]) {
                const int32_t trip = items[(size_t)s * kWave].n;
                S.slice_trip.push_back(trip);
                S.slice_arc.push_back((int64_t)S.arcs.size());
                const size_t first = (size_t)s * kWave;
                for (int lane = 0; lane < kWave; ++lane) {
                    const bool live = first + lane < items.size();
                    S.row_out.push_back(live ? items[first + lane].out : -1);
                    S.row_vidx.push_back(live ? items[first + lane].vidx : 0);
                }
                for (int32_t it = 0; it < trip; ++it)
                    for (int lane = 0; lane < kWave; ++lane) {
                        Arc a{0, pad_w};
                        if (first + lane < items.size() && it < items[first + lane].n) {
                            const int64_t e = items[first + lane].begin + it;
                            a.src = pcol[e];
                            a.w = pw[e];
                        }
                        S.arcs.push_back(a);
                    }
            }
        }
        ++n_levels;
        rows.swap(next_rows);
        pcol.swap(ncol);
        pw.swap(nwgt);
    }
    S.wave_ptr.push_back((int32_t)S.slice_trip.size());   // end of the last (level, wave) range
    sd.n_levels = n_levels;
    sd.n_part = n_part;
    S.max_part = std::max(S.max_part, n_part);
    S.sub.push_back(sd);
}

}  // namespace fb

namespace fb {

// Every index a kernel will dereference while walking the schedule stays inside
// the arrays it indexes.  n_out: number of targets of final rows, n_vidx: entries of
// the staged emission vector; a negative value means "the sub-graph's own state count".
bool sell_in_bounds(const SellHost &S, int32_t n_out, int32_t n_vidx, std::string &why)
{
    const size_t n_slices = S.slice_trip.size();
    if (S.slice_arc.size() != n_slices || S.row_out.size() != n_slices * kWave || S.row_vidx.size() != n_slices * kWave) {
        why = "slice arrays disagree in size";
        return false;
    }
    for (const SubDesc &sd : S.sub) {
        const size_t need = (size_t)sd.wave_ptr0 + (size_t)sd.n_levels * S.nw + 1;
        if (sd.wave_ptr0 < 0 || need > S.wave_ptr.size()) { why = "wave_ptr range"; return false; }
        for (int32_t l = 0; l < sd.n_levels; ++l)
            for (int wv = 0; wv < S.nw; ++wv) {
                const int32_t s0 = S.wave_ptr[(size_t)sd.wave_ptr0 + l * S.nw + wv];
                const int32_t s1 = S.wave_ptr[(size_t)sd.wave_ptr0 + l * S.nw + wv + 1];
                if (s0 < 0 || s1 < s0 || (size_t)s1 > n_slices) { why = "slice range"; return false; }
                for (int32_t s = s0; s < s1; ++s) {
                    const int32_t trip = S.slice_trip[s];
                    if (trip < 0 || trip > kChunk) { why = "trip count"; return false; }
                    if (S.slice_arc[s] < 0 || (size_t)S.slice_arc[s] + (size_t)trip * kWave > S.arcs.size()) {
                        why = "arc range";
                        return false;
                    }
                    const int32_t src_lim = l == 0 ? sd.K : sd.n_part;
                    for (size_t a = (size_t)S.slice_arc[s]; a < (size_t)S.slice_arc[s] + (size_t)trip * kWave; ++a)
                        if (S.arcs[a].src < 0 || S.arcs[a].src >= std::max(src_lim, 1)) { why = "arc source"; return false; }
                    for (int lane = 0; lane < kWave; ++lane) {
                        const int32_t o = S.row_out[(size_t)s * kWave + lane], v = S.row_vidx[(size_t)s * kWave + lane];
                        if (o >= (n_out < 0 ? sd.K : n_out) || (o < -1 && -2 - o >= sd.n_part)) { why = "row target"; return false; }
                        if (v < 0 || v >= std::max(n_vidx < 0 ? sd.K : n_vidx, 1)) { why = "emission index"; return false; }
                    }
                }
            }
    }
    return true;
}

// The schedule of sub-graph `sub` applied on the host in double precision, in the
// log semifield (log_semiring) or in ordinary arithmetic: y[out] for every final
// row, exactly as the kernels walk it (levels, slices, lanes), without the
// emission / offset step.  y must hold n_out doubles and is pre-filled by the caller.
void sell_apply_host(const SellHost &S, int32_t sub, bool log_semiring, const double *x, double *y)
{
    const SubDesc &sd = S.sub[(size_t)sub];
    std::vector<double> part((size_t)std::max(sd.n_part, 1), 0.0);
    for (int32_t l = 0; l < sd.n_levels; ++l) {
        const double *v = l == 0 ? x : part.data();
        std::vector<std::pair<int32_t, double>> writes;   // a level reads partials of the previous one only
        for (int wv = 0; wv < S.nw; ++wv) {
            const int32_t s0 = S.wave_ptr[(size_t)sd.wave_ptr0 + l * S.nw + wv];
            const int32_t s1 = S.wave_ptr[(size_t)sd.wave_ptr0 + l * S.nw + wv + 1];
            for (int32_t s = s0; s < s1; ++s)
                for (int lane = 0; lane < kWave; ++lane) {
                    const int32_t o = S.row_out[(size_t)s * kWave + lane];
                    if (o == -1) continue;
                    double m = -INFINITY, acc = 0.0;
                    for (int32_t it = 0; it < S.slice_trip[s]; ++it) {
                        const Arc &a = S.arcs[(size_t)S.slice_arc[s] + (size_t)it * kWave + lane];
                        if (log_semiring) m = std::max(m, (double)a.w + v[a.src]);
                        else acc += (double)a.w * v[a.src];
                    }
                    if (log_semiring) {
                        if (m == -INFINITY) acc = -INFINITY;
                        else {
                            for (int32_t it = 0; it < S.slice_trip[s]; ++it) {
                                const Arc &a = S.arcs[(size_t)S.slice_arc[s] + (size_t)it * kWave + lane];
                                acc += std::exp2((double)a.w + v[a.src] - m);
                            }
                            acc = m + std::log2(acc);
                        }
                    }
                    if (o >= 0) y[o] = acc;
                    else writes.emplace_back(-2 - o, acc);
                }
        }
        for (auto &wr : writes) part[(size_t)wr.first] = wr.second;
    }
}

}  // namespace fb
