// Host-side construction of the plan the probability-domain recursion kernel walks ("P-stream"), its
// interpretation on the host for tests, and the model of on-chip memory bank conflicts that its arc
// order is chosen by.
//
// The product is the same sparse matrix x vector product as in fb_sell.cpp (Eq. 4-5: row j gathers the
// arcs that enter, or leave, state j), for one shared graph and one workgroup of kNWShared waves, in
// ordinary arithmetic: the stream carries 2^w.
//
// Shape of the plan.
//   * A slice is 64 lanes walking arcs in lockstep.  A row of up to kPChunk arcs takes one lane, a longer
//     one 2, 4, ... 64 lanes of one slice (all rows of a slice take the same number of lanes, the kernel
//     adds the lanes of a row up when the slice ends); a row too long even for 64 lanes is cloned as in
//     fb_sell.cpp.  Rows are sorted by length; rows without arcs of non-zero weight are left out.
//   * Arcs travel in pairs: a unit is, per lane, three 32-bit words {source of arc 0 | source of arc 1 << 16,
//     2^w of arc 0, 2^w of arc 1} (6 bytes per arc), sources being byte offsets into the state buffer.  A
//     slice is a whole number of units (its lanes are padded with arcs of weight 0), and a wave's time step
//     is the units of its slices one after the other.  Of a wave's first kPPatterned units kPResident stay
//     in registers for the whole time loop (which ones: p_streamed), the rest is re-read from L2 every step.
//   * When a slice ends, every lane holds a row's sum (or a share of it) and needs to know where it goes and
//     which emission it takes: one 32-bit "close word" per lane and slice {target byte offset | emission
//     byte offset << 16}, kept in registers too (at most kPMaxClose slices per wave).  Which units end a
//     slice, and over how many lanes its rows are spread, is wave-uniform: a bit mask and a 3-bit field per
//     slice in the wave's descriptor.
//
// Bank conflicts.  The state vector lives in on-chip memory with 32 banks of 4 bytes; a 64-lane gather is
// served as two halves of 32 lanes, each taking as many cycles as the busiest bank has distinct addresses.
// With arcs in arbitrary order a gather takes about three times the two cycles it needs.  Which lane walks
// which row, and in which order a lane walks its arcs, is free, so both are chosen to spread every half's
// addresses of a step over the banks: rows are first traded between the halves of slices that both rows fit
// until no bank of a half serves more arcs than the slice has steps (as far as that goes), then each half's
// arcs are given their steps by an edge colouring of the graph lanes x banks (order_half).
#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>

#include "fb_internal.h"

namespace fb {

namespace {

constexpr int kBanks = 32, kHalf = 32;
constexpr double kPLastSimdShare = 1.0;

inline int bank_of(int32_t state) { return state & (kBanks - 1); }

struct PItem {
    int32_t out;               // target: state, or K + clone slot
    int32_t vidx;              // its emission index
    std::vector<int32_t> col;  // sources (state, or K + clone slot)
    std::vector<float> w;      // 2^w
};

int lanes_log2(int64_t n)
{
    int lg = 0;
    while (lg < 6 && (n + (1 << lg) - 1) / (1 << lg) > kPChunk) ++lg;
    return lg;
}

struct PSlice {
    int lg = 0;
    int trip = 0;                 // arcs per lane (even)
    std::vector<int32_t> items;   // indices into the item list, at most 64 >> lg
};

// cycles one half of a gather takes: the largest number of distinct addresses any bank has to serve (at least 1)
int half_cycles(const int32_t *addr, int n)
{
    int32_t seen[kHalf];
    int cnt[kBanks] = {};
    int ns = 0, worst = 1;
    for (int i = 0; i < n; ++i) {
        bool dup = false;
        for (int j = 0; j < ns; ++j) dup = dup || seen[j] == addr[i];
        if (dup) continue;
        seen[ns++] = addr[i];
        worst = std::max(worst, ++cnt[bank_of(addr[i])]);
    }
    return worst;
}

// Lays out the arcs of one half of a slice.  lanes: for every lane of the half the arcs it has to walk (any order),
// at most trip each.  Returns, per lane, the arcs in walking order, padded to trip with {-1, 0} entries (the caller
// gives those an address that costs nothing).  A gather is free of conflicts when its lanes read different banks, so
// an order is an edge colouring of the bipartite multigraph lanes x banks (an arc = an edge from its lane to the bank
// of its source, a colour = a step): with as many colours as the largest degree such a colouring always exists
// (Koenig), and it is found edge by edge, an alternating path recoloured where the two ends have no free colour in
// common.  A bank that serves more arcs than there are steps is split into as many nodes as it needs to bring every
// node's degree down to the number of steps: then a step has at most that many arcs of the bank, which is the least
// any order could do.
void order_half_coloured(const std::vector<std::vector<std::pair<int32_t, float>>> &lanes, int trip,
                         std::vector<std::vector<std::pair<int32_t, float>>> &out)
{
    const int nl = (int)lanes.size();
    struct Edge { int lane, node, idx; };
    std::vector<Edge> edges;
    int bank_deg[kBanks] = {}, parts[kBanks], first_node[kBanks], seen[kBanks] = {};
    for (int u = 0; u < nl; ++u)
        for (const auto &a : lanes[u]) ++bank_deg[bank_of(a.first)];
    int n_nodes = 0;
    for (int bk = 0; bk < kBanks; ++bk) {
        parts[bk] = std::max(1, (bank_deg[bk] + trip - 1) / trip);
        first_node[bk] = n_nodes;
        n_nodes += parts[bk];
    }
    for (int u = 0; u < nl; ++u)
        for (int i = 0; i < (int)lanes[u].size(); ++i) {
            const int bk = bank_of(lanes[u][i].first);
            edges.push_back({u, first_node[bk] + seen[bk]++ / trip, i});   // (node after node filled: only the surplus shares a step)
        }
    // the arcs of the surplus nodes first: they take the lowest colours, so that the surplus of different banks meets in
    // the same few steps instead of spoiling a step each
    std::stable_sort(edges.begin(), edges.end(), [&](const Edge &x, const Edge &y) {
        const bool sx = x.node != first_node[bank_of(lanes[(size_t)x.lane][(size_t)x.idx].first)];
        const bool sy = y.node != first_node[bank_of(lanes[(size_t)y.lane][(size_t)y.idx].first)];
        return sx && !sy;
    });
    const int n_col = trip;
    std::vector<int> at_lane((size_t)nl * n_col, -1), at_node((size_t)n_nodes * n_col, -1), colour(edges.size(), -1);
    auto free_at = [&](const std::vector<int> &tab, int v) {
        for (int c = 0; c < n_col; ++c)
            if (tab[(size_t)v * n_col + c] < 0) return c;
        return -1;
    };
    for (int e = 0; e < (int)edges.size(); ++e) {
        const int u = edges[e].lane, v = edges[e].node;
        const int a = free_at(at_lane, u), b = free_at(at_node, v);   // (both exist: no degree is above n_col)
        if (at_node[(size_t)v * n_col + a] >= 0) {
            // a is taken at the bank: walk from the bank along colours a, b, a, ... and swap the two on that path (it
            // cannot come back to lane u, which has no edge of colour a)
            std::vector<int> path;
            int x = v, c = a;
            bool on_node = true;
            for (;;) {
                const int f = on_node ? at_node[(size_t)x * n_col + c] : at_lane[(size_t)x * n_col + c];
                if (f < 0) break;
                path.push_back(f);
                x = on_node ? edges[f].lane : edges[f].node;
                on_node = !on_node;
                c = c == a ? b : a;
            }
            for (int f : path) {
                at_lane[(size_t)edges[f].lane * n_col + colour[f]] = -1;
                at_node[(size_t)edges[f].node * n_col + colour[f]] = -1;
            }
            for (int f : path) {
                colour[f] = colour[f] == a ? b : a;
                at_lane[(size_t)edges[f].lane * n_col + colour[f]] = f;
                at_node[(size_t)edges[f].node * n_col + colour[f]] = f;
            }
        }
        colour[e] = a;
        at_lane[(size_t)u * n_col + a] = e;
        at_node[(size_t)v * n_col + a] = e;
    }
    out.assign((size_t)nl, std::vector<std::pair<int32_t, float>>((size_t)trip, {-1, 0.0f}));
    for (int e = 0; e < (int)edges.size(); ++e) out[(size_t)edges[e].lane][(size_t)colour[e]] = lanes[(size_t)edges[e].lane][(size_t)edges[e].idx];
}

// The same by a greedy rule: step by step, the banks that still have the most to serve are served first, and several
// lanes that read one address count once (which the colouring does not know about: where many lanes read the same
// states, this order is the better one).
void order_half_greedy(const std::vector<std::vector<std::pair<int32_t, float>>> &lanes, int trip,
                std::vector<std::vector<std::pair<int32_t, float>>> &out)
{
    const int nl = (int)lanes.size();
    std::vector<std::vector<std::pair<int32_t, float>>> rem = lanes;
    out.assign((size_t)nl, {});
    for (int t = 0; t < trip; ++t) {
        const int need = trip - t;   // a lane with this many arcs left has no step to spare
        int load[kBanks] = {};
        for (const auto &l : rem)
            for (const auto &a : l) ++load[bank_of(a.first)];
        int32_t used_addr[kBanks];
        bool used[kBanks] = {};
        // lanes without slack first, then those with the fewest banks to choose from
        std::vector<int> order((size_t)nl);
        std::iota(order.begin(), order.end(), 0);
        std::vector<int> n_banks((size_t)nl, 0);
        for (int u = 0; u < nl; ++u) {
            bool b[kBanks] = {};
            for (const auto &a : rem[u]) b[bank_of(a.first)] = true;
            for (int i = 0; i < kBanks; ++i) n_banks[u] += b[i] ? 1 : 0;
        }
        std::stable_sort(order.begin(), order.end(), [&](int x, int y) {
            const bool mx = (int)rem[x].size() >= need, my = (int)rem[y].size() >= need;
            if (mx != my) return mx;
            return n_banks[x] < n_banks[y];
        });
        std::vector<int> pick((size_t)nl, -1);
        for (int u : order) {
            if (rem[u].empty()) continue;
            const bool must = (int)rem[u].size() >= need;
            int best = -1;
            long best_score = -1;
            for (int i = 0; i < (int)rem[u].size(); ++i) {
                const int32_t a = rem[u][i].first;
                const int bk = bank_of(a);
                long score;
                if (used[bk]) score = used_addr[bk] == a ? 3000000L + load[bk] : 1000L - load[bk];   // same address: free; else a conflict
                else score = 2000000L + load[bk];
                if (score > best_score) { best_score = score; best = i; }
            }
            if (best_score < 2000000L && !must) continue;   // wait rather than collide
            pick[u] = best;
            const int32_t a = rem[u][best].first;
            if (!used[bank_of(a)]) { used[bank_of(a)] = true; used_addr[bank_of(a)] = a; }
        }
        for (int u = 0; u < nl; ++u) {
            if (pick[u] < 0) {
                out[u].push_back({-1, 0.0f});
            } else {
                out[u].push_back(rem[u][pick[u]]);
                rem[u].erase(rem[u].begin() + pick[u]);
            }
        }
    }
}

// gather cycles of a laid-out half under the bank model (padding entries cost nothing)
long laid_cycles(const std::vector<std::vector<std::pair<int32_t, float>>> &laid, int trip)
{
    long cyc = 0;
    for (int t = 0; t < trip; ++t) {
        int32_t addr[kHalf];
        int n = 0;
        for (const auto &l : laid)
            if (l[(size_t)t].first >= 0) addr[n++] = l[(size_t)t].first;
        cyc += half_cycles(addr, n);
    }
    return cyc;
}

// the better of the two orders
void order_half(const std::vector<std::vector<std::pair<int32_t, float>>> &lanes, int trip,
                std::vector<std::vector<std::pair<int32_t, float>>> &out)
{
    std::vector<std::vector<std::pair<int32_t, float>>> other;
    order_half_coloured(lanes, trip, out);
    if (laid_cycles(out, trip) == trip) return;   // (nothing to gain)
    order_half_greedy(lanes, trip, other);
    if (laid_cycles(other, trip) < laid_cycles(out, trip)) out.swap(other);
}

}  // namespace

bool pstream_build(int32_t K, const int64_t *ptr, const int32_t *col, const float *w, const int32_t *row_vidx, int32_t n_vidx,
                   PStreamHost &S, std::string &why)
{
    const int nw = kNWShared - 1;
    S = PStreamHost();
    S.K = K;
    if (K + 1 > kXsFixed) { why = "more states than the fixed buffers hold"; return false; }
    if (n_vidx + 1 > 0x3fff) { why = "emission index beyond 14 bits"; return false; }

    // ---- rows that need clones (as in fb_sell.cpp): counted on the arcs of non-zero weight
    const int64_t row_cap = (int64_t)kWave * kPChunk;
    std::vector<int64_t> n_live((size_t)K, 0);
    for (int32_t r = 0; r < K; ++r)
        for (int64_t e = ptr[r]; e < ptr[r + 1]; ++e) n_live[r] += w[e] > -INFINITY ? 1 : 0;
    // a cloned source repeats the arcs that leave it, which makes rows longer: settle the clone counts first
    std::vector<int32_t> n_share((size_t)K, 1), first_slot((size_t)K, 0);
    for (int round = 0; round < 8; ++round) {
        bool changed = false;
        for (int32_t r = 0; r < K; ++r) {
            int64_t n = 0;
            for (int64_t e = ptr[r]; e < ptr[r + 1]; ++e)
                if (w[e] > -INFINITY) n += n_share[col[e]];
            const int32_t s = (int32_t)std::max<int64_t>(1, (n + row_cap - 1) / row_cap);
            if (s > n_share[r]) { n_share[r] = s; changed = true; }
        }
        if (!changed) break;
    }
    int32_t n_slot = 0;
    for (int32_t r = 0; r < K; ++r) {
        if (n_share[r] <= 1) continue;
        first_slot[r] = n_slot;
        S.clones.push_back(CloneDesc{r, n_slot, n_share[r] - 1, 0});
        n_slot += n_share[r] - 1;
    }
    S.Ccap = n_slot;
    if (K + n_slot + 1 > kXsFixed) { why = "states and clone slots exceed the fixed buffers"; return false; }
    const int32_t dump = K + n_slot;

    // ---- items: one per row or clone, arcs of weight zero dropped, arcs out of cloned states repeated
    std::vector<PItem> items;
    double w_min = INFINITY, row_top = 0.0;
    for (int32_t r = 0; r < K; ++r) {
        std::vector<int32_t> pc;
        std::vector<float> pw;
        double rsum = 0.0;
        for (int64_t e = ptr[r]; e < ptr[r + 1]; ++e) {
            if (!(w[e] > -INFINITY)) continue;
            if (!(w[e] >= -kLinWeightSpan && w[e] <= kLinRowSumTop)) { why = "an arc weight outside the range of the probability-domain kernel"; return false; }
            const float W = exp2f(w[e]);
            w_min = std::min(w_min, (double)W);
            for (int32_t c = 0; c < n_share[col[e]]; ++c) {
                pc.push_back(c == 0 ? col[e] : K + first_slot[col[e]] + c - 1);
                pw.push_back(W);
                rsum += (double)W;
            }
        }
        row_top = std::max(row_top, rsum);
        if (pc.empty()) {
            S.zero_rows.push_back(r);
            continue;
        }
        const int32_t shares = n_share[r];
        const int64_t n = (int64_t)pc.size();
        int64_t at = 0;
        for (int32_t c = 0; c < shares; ++c) {
            const int64_t len = n / shares + (c < n % shares ? 1 : 0);
            PItem it;
            it.out = c == 0 ? r : K + first_slot[r] + c - 1;
            it.vidx = row_vidx[r];
            it.col.assign(pc.begin() + at, pc.begin() + at + len);
            it.w.assign(pw.begin() + at, pw.begin() + at + len);
            at += len;
            if (len > 0) items.push_back(std::move(it));
            else S.zero_rows.push_back(it.out);   // (cannot happen: shares <= arcs)
        }
    }
    // scale and range guard of the kernel (see linear_run): entries stay below 2^(bias + 1 + r2), row sums below 2^(bias + 1 + 2 r2)
    {
        const int r2 = (int)std::ceil(std::log2(std::max(row_top, 1.0)));
        const int w2 = w_min < 1.0 ? (int)std::floor(std::log2(w_min)) : 0;
        S.bias = 122 - 2 * r2;
        if (S.bias < 24) { why = "rows whose weights add up to too much for the probability-domain kernel"; return false; }
        S.dim = (float)std::exp2((double)(-124 - w2));
    }

    // ---- slices: longest rows first; a slice takes its lanes per row from its first (longest) row
    std::vector<int32_t> order(items.size());
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return items[a].col.size() > items[b].col.size(); });
    std::vector<PSlice> slices;
    for (size_t i = 0; i < order.size();) {
        PSlice sl;
        const int64_t n0 = (int64_t)items[order[i]].col.size();
        sl.lg = lanes_log2(n0);
        const int count = (int)std::min<size_t>((size_t)(kWave >> sl.lg), order.size() - i);
        sl.trip = (int)((n0 + (1 << sl.lg) - 1) >> sl.lg);
        sl.trip += sl.trip & 1;
        for (int j = 0; j < count; ++j) sl.items.push_back(order[i + j]);
        slices.push_back(std::move(sl));
        i += (size_t)count;
    }

    // ---- trade rows between the halves of slices that both rows fit until each half's arcs are spread evenly over the banks
    // (one lane per row only: the rows of a slice of wider rows share their half anyway)
    {
        auto half_hist = [&](const PSlice &sl, int h, int *hist) {
            std::fill(hist, hist + kBanks, 0);
            for (int j = h * kHalf; j < std::min<int>((h + 1) * kHalf, (int)sl.items.size()); ++j)
                for (int32_t c : items[sl.items[j]].col) ++hist[bank_of(c)];
        };
        auto peak = [&](const int *hist) { return *std::max_element(hist, hist + kBanks); };
        // groups of (slice, half) with the same trip and one lane per row
        std::vector<std::pair<int, int>> halves;
        for (int s = 0; s < (int)slices.size(); ++s)
            if (slices[s].lg == 0)
                for (int h = 0; h * kHalf < (int)slices[s].items.size(); ++h) halves.push_back({s, h});
        uint64_t rng = 0x9E3779B97F4A7C15ull;
        auto next = [&]() { rng ^= rng << 13; rng ^= rng >> 7; rng ^= rng << 17; return rng; };
        std::vector<std::vector<int>> hist(halves.size(), std::vector<int>(kBanks));
        for (size_t i = 0; i < halves.size(); ++i) half_hist(slices[halves[i].first], halves[i].second, hist[i].data());
        const int64_t tries = std::min<int64_t>(400000, 200 * (int64_t)items.size());
        for (int64_t it = 0; it < tries && halves.size() > 1; ++it) {
            const size_t a = (size_t)(next() % halves.size());
            // a partner nearby: halves are in slice order, slices of similar trips are neighbours
            const int span = 12;
            const size_t lo = a > (size_t)span ? a - span : 0, hi = std::min(halves.size() - 1, a + span);
            const size_t b2 = lo + (size_t)(next() % (hi - lo + 1));
            if (b2 == a) continue;
            PSlice &sa = slices[halves[a].first], &sb = slices[halves[b2].first];
            const int na = std::min<int>(kHalf, (int)sa.items.size() - halves[a].second * kHalf);
            const int nb = std::min<int>(kHalf, (int)sb.items.size() - halves[b2].second * kHalf);
            const int ia = halves[a].second * kHalf + (int)(next() % (uint64_t)na), ib = halves[b2].second * kHalf + (int)(next() % (uint64_t)nb);
            const PItem &ra = items[sa.items[ia]], &rb = items[sb.items[ib]];
            if ((int)ra.col.size() > sb.trip || (int)rb.col.size() > sa.trip) continue;   // each row must fit the other slice
            // what the two halves cost before and after the swap: a half whose fullest bank serves no more arcs than
            // the slice has steps can be walked without conflicts, the surplus is what counts
            std::vector<int> &ha = hist[a], &hb = hist[b2];
            auto cost = [&]() { return std::max(peak(ha.data()), sa.trip) + std::max(peak(hb.data()), sb.trip); };
            const int before = cost();
            long sq_before = 0, sq_after = 0;
            for (int k = 0; k < kBanks; ++k) sq_before += (long)ha[k] * ha[k] + (long)hb[k] * hb[k];
            for (int32_t c : ra.col) { --ha[bank_of(c)]; ++hb[bank_of(c)]; }
            for (int32_t c : rb.col) { ++ha[bank_of(c)]; --hb[bank_of(c)]; }
            const int after = cost();
            for (int k = 0; k < kBanks; ++k) sq_after += (long)ha[k] * ha[k] + (long)hb[k] * hb[k];
            if (after < before || (after == before && sq_after < sq_before)) {
                std::swap(sa.items[ia], sb.items[ib]);
            } else {   // undo
                for (int32_t c : ra.col) { ++ha[bank_of(c)]; --hb[bank_of(c)]; }
                for (int32_t c : rb.col) { --ha[bank_of(c)]; ++hb[bank_of(c)]; }
            }
        }
    }

    // ---- deal slices to the waves: most units first, to the wave that would finish first and still has a close word free
    std::vector<int> sorder(slices.size());
    std::iota(sorder.begin(), sorder.end(), 0);
    std::stable_sort(sorder.begin(), sorder.end(), [&](int a, int b) { return slices[a].trip > slices[b].trip; });
    std::vector<std::vector<int>> mine((size_t)nw);
    std::vector<int64_t> load((size_t)nw, 0);
    for (int s : sorder) {
        // (waves go round the four SIMDs of a compute unit; the last SIMD hosts the data-moving wave in place of a fourth
        // arc-walking one, so its three arc-walking waves get more of its issue slots and take more units)
        auto finish = [&](int wv) { return (double)(load[wv] + slices[s].trip / 2) / (wv % 4 == 3 ? kPLastSimdShare : 1.0); };
        int best = -1;
        for (int wv = 0; wv < nw; ++wv)
            if ((int)mine[wv].size() < kPMaxClose && (best < 0 || finish(wv) < finish(best))) best = wv;
        if (best < 0) { why = "more slices than the waves have close words for"; return false; }
        mine[best].push_back(s);
        load[best] += slices[s].trip / 2;
    }

    // ---- emit
    const uint32_t dump_off = (uint32_t)dump * 4u;
    S.waves.resize((size_t)nw);
    for (int wv = 0; wv < nw; ++wv) {
        PWaveDesc &wd = S.waves[wv];
        std::memset(&wd, 0, sizeof(wd));
        wd.unit_base = (int64_t)(S.units.size() / (3 * kWave));
        wd.cw_base = (int32_t)(S.close_words.size() / kWave);
        int32_t n_units = 0, n_close = 0;
        for (int s : mine[wv]) {
            const PSlice &sl = slices[s];
            const int g = 1 << sl.lg, trip = sl.trip;
            // the arcs every lane has to walk: a row's arcs are dealt to its g lanes (a row over both halves: bank by
            // bank alternately, so that each half gets half of every bank's share)
            std::vector<std::vector<std::pair<int32_t, float>>> lanes((size_t)kWave);
            for (int j = 0; j < (int)sl.items.size(); ++j) {
                const PItem &im = items[sl.items[j]];
                std::vector<int> idx(im.col.size());
                std::iota(idx.begin(), idx.end(), 0);
                if (g > 1) std::stable_sort(idx.begin(), idx.end(), [&](int a, int b) { return bank_of(im.col[a]) < bank_of(im.col[b]); });
                for (size_t q = 0; q < idx.size(); ++q) {
                    // lanes of the row in turn, the two halves of a 64-lane row alternating
                    const int t = (int)(q % (size_t)g);
                    const int lane_in_row = g == kWave ? ((t & 1) * kHalf + (t >> 1)) : t;
                    lanes[(size_t)(j * g + lane_in_row)].push_back({im.col[idx[q]], im.w[idx[q]]});
                }
            }
            for (int l = 0; l < kWave; ++l)
                if ((int)lanes[l].size() > trip) { why = "internal error: a lane with more arcs than its slice walks"; return false; }
            std::vector<std::vector<std::pair<int32_t, float>>> laid((size_t)kWave);
            for (int h = 0; h < 2; ++h) {
                std::vector<std::vector<std::pair<int32_t, float>>> in(lanes.begin() + h * kHalf, lanes.begin() + (h + 1) * kHalf), out;
                order_half(in, trip, out);
                for (int l = 0; l < kHalf; ++l) laid[(size_t)(h * kHalf + l)] = std::move(out[l]);
            }
            // padding entries (weight 0) read what a lane of their half reads in the same step, or the lane's own bank
            for (int t = 0; t < trip; ++t)
                for (int h = 0; h < 2; ++h) {
                    int32_t any = -1;
                    for (int l = h * kHalf; l < (h + 1) * kHalf; ++l)
                        if (laid[l][t].first >= 0) { any = laid[l][t].first; break; }
                    for (int l = h * kHalf; l < (h + 1) * kHalf; ++l)
                        if (laid[l][t].first < 0) laid[l][t] = {any >= 0 ? any : std::min(l - h * kHalf, K - 1), 0.0f};
                }
            for (int u = 0; u < trip / 2; ++u)
                for (int l = 0; l < kWave; ++l) {
                    const auto &a0 = laid[l][2 * u], &a1 = laid[l][2 * u + 1];
                    S.units.push_back((uint32_t)a0.first * 4u | ((uint32_t)a1.first * 4u) << 16);
                    uint32_t b0, b1;
                    std::memcpy(&b0, &a0.second, 4);
                    std::memcpy(&b1, &a1.second, 4);
                    S.units.push_back(b0);
                    S.units.push_back(b1);
                }
            for (int l = 0; l < kWave; ++l) {
                const int j = l >> sl.lg;
                if (j < (int)sl.items.size()) {
                    const PItem &im = items[sl.items[j]];
                    S.close_words.push_back((uint32_t)im.out * 4u | ((uint32_t)im.vidx * 4u) << 16);
                } else {
                    S.close_words.push_back(dump_off | ((uint32_t)n_vidx * 4u) << 16);   // nothing: the dump slot, the emission that is zero
                }
            }
            n_units += trip / 2;
            if (n_units > kPMaxUnits) { why = "more arcs per wave and time step than the kernel's unit masks cover"; return false; }
            wd.close_mask[(n_units - 1) / 64] |= (uint64_t)1 << ((n_units - 1) % 64);
            wd.lgs |= (uint64_t)sl.lg << (3 * n_close);
            ++n_close;
        }
        if (n_units > kPMaxUnits) { why = "more arcs per wave and time step than the kernel's unit masks cover"; return false; }
        wd.n_units = n_units;
        wd.n_close = n_close;
    }
    // the kernel loads whole groups of resident units and close words whatever a wave's count: room behind the last
    S.units.resize(S.units.size() + (size_t)kPPatterned * 3 * kWave, 0u);
    S.close_words.resize(S.close_words.size() + (size_t)kPMaxClose * kWave, dump_off | ((uint32_t)n_vidx * 4u) << 16);
    return true;
}

// Everything the kernel will index while walking the plan stays in range.
bool pstream_in_bounds(const PStreamHost &S, int32_t n_vidx, std::string &why)
{
    const size_t n_units_total = S.units.size() / (3 * kWave), n_cw_total = S.close_words.size() / kWave;
    if (S.waves.size() != (size_t)(kNWShared - 1)) { why = "wave count"; return false; }
    if (S.K + S.Ccap + 1 > kXsFixed) { why = "index space"; return false; }
    const uint32_t top = (uint32_t)(S.K + S.Ccap) * 4u;   // the dump slot's offset: the largest a source or target may have
    for (const PWaveDesc &wd : S.waves) {
        if (wd.n_units < 0 || wd.n_units > kPMaxUnits || wd.n_close < 0 || wd.n_close > kPMaxClose) { why = "unit or close count"; return false; }
        if (wd.unit_base < 0 || (size_t)wd.unit_base + (size_t)std::max(wd.n_units, kPPatterned) > n_units_total) { why = "unit range"; return false; }
        if (wd.cw_base < 0 || (size_t)wd.cw_base + (size_t)kPMaxClose > n_cw_total) { why = "close word range"; return false; }
        int closes = 0;
        for (int u = 0; u < kPMaxUnits; ++u) {
            const bool c = (wd.close_mask[u / 64] >> (u % 64)) & 1u;
            if (c && u >= wd.n_units) { why = "close behind the last unit"; return false; }
            closes += c ? 1 : 0;
        }
        if (closes != wd.n_close) { why = "close mask and count disagree"; return false; }
        if (wd.n_units > 0 && !((wd.close_mask[(wd.n_units - 1) / 64] >> ((wd.n_units - 1) % 64)) & 1u)) { why = "last unit does not close"; return false; }
        for (size_t i = (size_t)wd.unit_base * 3 * kWave; i < ((size_t)wd.unit_base + (size_t)wd.n_units) * 3 * kWave; i += 3) {
            const uint32_t s = S.units[i];
            if ((s & 0xffffu) > top || (s >> 16) > top || (s & 3u) || ((s >> 16) & 3u)) { why = "arc source"; return false; }
            float w0, w1;
            std::memcpy(&w0, &S.units[i + 1], 4);
            std::memcpy(&w1, &S.units[i + 2], 4);
            if (!(w0 >= 0.0f && w0 < INFINITY && w1 >= 0.0f && w1 < INFINITY)) { why = "arc weight"; return false; }
        }
        for (size_t i = (size_t)wd.cw_base * kWave; i < ((size_t)wd.cw_base + (size_t)wd.n_close) * kWave; ++i) {
            const uint32_t cw = S.close_words[i];
            if ((cw & 0xffffu) > top || (cw & 3u) || (cw >> 16) > (uint32_t)n_vidx * 4u || ((cw >> 16) & 3u)) { why = "close word"; return false; }
            if ((cw & 0xffffu) == top && (cw >> 16) != (uint32_t)n_vidx * 4u) { why = "emission on the dump slot"; return false; }
        }
    }
    for (const CloneDesc &cd : S.clones)
        if (cd.state < 0 || cd.state >= S.K || cd.first < 0 || cd.count < 1 || cd.first + cd.count > S.Ccap) { why = "clone entry"; return false; }
    for (int32_t z : S.zero_rows)
        if (z < 0 || z >= S.K + S.Ccap) { why = "zero row"; return false; }
    return true;
}

// y = A x as the kernel forms it (lanes, groups of lanes, clones), in double; x and y hold one value per state
// (ordinary numbers, not logs).  cycles (nullable): the gather cycles of a time step under the bank model above,
// and the least any order could need (two per gather).
bool pstream_apply_host(const PStreamHost &S, const double *x, double *y, int64_t *cycles, int64_t *cycles_floor, std::string &why)
{
    std::vector<double> xe((size_t)S.K + (size_t)S.Ccap + 1, 0.0), ye((size_t)S.K + (size_t)S.Ccap + 1, 0.0);
    for (int32_t k = 0; k < S.K; ++k) xe[k] = x[k];   // a cloned state's value sits in the state itself, its clones hold zero
    int64_t cyc = 0, floor_cyc = 0;
    for (const PWaveDesc &wd : S.waves) {
        double acc[kWave] = {};
        int c = 0;
        for (int u = 0; u < wd.n_units; ++u) {
            const uint32_t *unit = S.units.data() + ((size_t)wd.unit_base + (size_t)u) * 3 * kWave;
            for (int r = 0; r < 2; ++r) {
                int32_t addr[kWave];
                for (int l = 0; l < kWave; ++l) {
                    const uint32_t s = unit[l * 3];
                    addr[l] = (int32_t)((r ? s >> 16 : s & 0xffffu) / 4u);
                    float wt;
                    std::memcpy(&wt, &unit[l * 3 + 1 + r], 4);
                    acc[l] += (double)wt * xe[(size_t)addr[l]];
                }
                cyc += half_cycles(addr, kHalf) + half_cycles(addr + kHalf, kHalf);
                floor_cyc += 2;
            }
            if ((wd.close_mask[u / 64] >> (u % 64)) & 1u) {
                const int g = 1 << ((wd.lgs >> (3 * c)) & 7u);
                const uint32_t *cw = S.close_words.data() + ((size_t)wd.cw_base + (size_t)c) * kWave;
                for (int l = 0; l < kWave; l += g) {
                    double tot = 0.0;
                    for (int t = 0; t < g; ++t) tot += acc[l + t];
                    for (int t = 0; t < g; ++t) {
                        const uint32_t tgt = (cw[l + t] & 0xffffu) / 4u;
                        if (tgt != (cw[l] & 0xffffu) / 4u) { why = "lanes of a row disagree about its target"; return false; }
                        if (tgt == (uint32_t)(S.K + S.Ccap) && tot != 0.0) { why = "a row's total goes to the dump slot"; return false; }
                        ye[tgt] = tot;
                        acc[l + t] = 0.0;
                    }
                }
                ++c;
            }
        }
    }
    for (const CloneDesc &cd : S.clones)
        for (int32_t i = 0; i < cd.count; ++i) ye[(size_t)cd.state] += ye[(size_t)S.K + (size_t)cd.first + i];
    for (int32_t k = 0; k < S.K; ++k) y[k] = ye[(size_t)k];
    if (cycles) *cycles = cyc;
    if (cycles_floor) *cycles_floor = floor_cyc;
    return true;
}

}  // namespace fb
