// Stream form of a log-semiring schedule (see fb_internal.h): built from the
// row-split sliced-ELL plan, checked for bounds, and interpreted on the host
// for tests of the scheduling logic.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <utility>

#include "fb_internal.h"

namespace fb {

namespace {

float bits_to_float(uint32_t u)
{
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

uint32_t float_to_bits(float f)
{
    uint32_t u;
    std::memcpy(&u, &f, 4);
    return u;
}

constexpr int kBatchEntries = kBatchRows * kWave;

// Position of (row r, lane) inside a batch: a lane reads two consecutive rows with one 16-byte load,
// so rows are stored in pairs, lane-major within a pair.
inline size_t entry_at(size_t batch, int r, int lane)
{
    return batch * kBatchEntries + (size_t)(r / 2) * (2 * kWave) + (size_t)lane * 2 + (size_t)(r % 2);
}

// flag byte of batch bt of a wave's step: resident batches first (two words), then the streamed ones
uint32_t batch_flags(const StreamHost &S, const WaveDesc &wd, size_t bt)
{
    if (bt < (size_t)kResident) return (S.flagwords[(size_t)wd.flag_base + bt / 4] >> (8 * (bt % 4))) & 0xffu;
    const size_t s = bt - kResident;
    return (S.flagwords[(size_t)wd.flag_base + 2 + s / kRing] >> (8 * (s % kRing))) & 0xffu;
}

size_t wave_batches(const WaveDesc &wd) { return (size_t)kResident + (size_t)wd.n_iter * kRing; }

}  // namespace

bool stream_from_sell(const SellHost &S, int32_t Kcap, int32_t Ecap, int32_t esize, StreamHost &out, std::string &why)
{
    out.nw = S.nw;
    out.esize = esize;
    out.Kcap = Kcap;
    out.Ccap = S.max_slot;
    out.Ecap = Ecap;
    out.clones = S.clones;
    out.zero_rows = S.zero_rows;
    if (((int64_t)Kcap + S.max_slot + 1) * esize > 0xffff || Ecap + 1 > 0xffff) {
        why = "state vector (with clone slots) beyond 64 KB, or emission entries beyond 16 bits";
        return false;
    }
    const uint32_t dump = (uint32_t)(Kcap + S.max_slot);
    const size_t xs = (size_t)dump + 1;
    const Arc pad_arc{0, -INFINITY};
    for (const SubDesc &ssd : S.sub) {
        SubDesc sd = ssd;
        sd.wave_ptr0 = (int32_t)out.waves.size();
        const size_t vix0 = out.vix.size();
        out.vix.resize(vix0 + xs, (uint16_t)Ecap);   // targets that are never written take the zero emission
        for (int wv = 0; wv < S.nw; ++wv) {
            WaveDesc wd{};
            wd.arc_base = (int64_t)out.arcs.size();
            std::vector<uint8_t> flags;   // one per batch
            std::vector<Arc> lin;         // the wave's rows in order, 64 entries each
            auto pad_batch = [&]() {   // zero-weight arcs whose sums go to the dump slot
                for (int e = 0; e < (kBatchRows - 1) * kWave; ++e) lin.push_back(pad_arc);
                for (int lane = 0; lane < kWave; ++lane) lin.push_back(Arc{(int32_t)(dump << 16), -INFINITY});
                flags.push_back((uint8_t)(kFlagInfo | kFlagSkip));
            };
            const int32_t s0 = S.wave_ptr[(size_t)ssd.wave_ptr0 + wv], s1 = S.wave_ptr[(size_t)ssd.wave_ptr0 + wv + 1];
            for (int32_t s = s0; s < s1; ++s) {
                const int32_t trip = S.slice_trip[s], stack = S.slice_stack[s];
                const int32_t nb = (trip + kBatchRows - 1) / kBatchRows, rows = nb * kBatchRows;
                const int32_t rows_per = stack ? kBatchRows / stack : rows;   // rows of one part of a lane
                if (stack && flags.size() >= (size_t)kMaxStacked) {
                    why = "stacked batch behind the first batches of a wave";
                    return false;
                }
                for (int32_t it = 0; it < rows; ++it)
                    for (int lane = 0; lane < kWave; ++lane) {
                        Arc a = it < trip ? S.arcs[(size_t)S.slice_arc[s] + (size_t)it * kWave + lane] : pad_arc;
                        if (a.src >= ssd.K) a.src = Kcap + (a.src - ssd.K);   // a clone: its slot in the state buffer
                        a.src *= esize;                                       // byte offset into the buffer
                        if (it % rows_per == rows_per - 1) {   // the last entry of a part also names the part's target
                            const size_t at = ((size_t)s * kWave + lane) * kBatchRows + (size_t)(it / rows_per);
                            const int32_t o = S.row_out[at], v = S.row_vidx[at];
                            const uint32_t tgt = o < 0 ? dump : (o < ssd.K ? (uint32_t)o : (uint32_t)(Kcap + (o - ssd.K)));
                            a.src = (int32_t)((uint32_t)a.src | (tgt << 16));
                            if (o >= 0) out.vix[vix0 + tgt] = (uint16_t)v;
                        }
                        lin.push_back(a);
                    }
                for (int32_t bt = 0; bt < nb; ++bt) {
                    uint32_t f = bt + 1 == nb ? (kFlagInfo | ((uint32_t)S.slice_lg[s] << kFlagLgShift)) : 0u;
                    if (stack == 2) f |= kFlagDual;
                    if (stack == kBatchRows) f |= kFlagQuad;
                    flags.push_back((uint8_t)f);
                }
            }
            while (flags.size() < (size_t)kResident || (flags.size() - kResident) % kRing) pad_batch();   // whole iterations
            if ((flags.size() - kResident) / kRing > 2 * kWave) {
                why = "more than " + std::to_string(2 * kWave * kRing * kBatchRows * kWave) + " arcs per wave and time step";
                return false;
            }
            out.arcs.resize((size_t)wd.arc_base + lin.size());
            for (size_t bt = 0; bt < flags.size(); ++bt)
                for (int r = 0; r < kBatchRows; ++r)
                    for (int lane = 0; lane < kWave; ++lane)
                        out.arcs[(size_t)wd.arc_base + entry_at(bt, r, lane)] = lin[(bt * kBatchRows + r) * kWave + lane];
            wd.n_iter = (int32_t)((flags.size() - kResident) / kRing);
            wd.flag_base = (int32_t)out.flagwords.size();
            for (int wi = 0; wi < 2; ++wi) {   // resident batches: two words, unused bytes say "skip"
                uint32_t wdw = 0;
                for (int j = 0; j < 4; ++j)
                    wdw |= (uint32_t)(wi * 4 + j < kResident ? flags[(size_t)wi * 4 + j] : (uint8_t)kFlagSkip) << (8 * j);
                out.flagwords.push_back(wdw);
            }
            for (size_t i = kResident; i < flags.size(); i += kRing) {
                uint32_t wdw = 0;
                for (int j = 0; j < kRing; ++j) wdw |= (uint32_t)flags[i + j] << (8 * j);
                out.flagwords.push_back(wdw);
            }
            out.waves.push_back(wd);
        }
        out.sub.push_back(sd);
    }
    return true;
}

// Everything the kernel will index while interpreting the streams stays in range.
// n_vidx: entries of the staged emission vector (negative: the sub-graph's state count).
bool stream_in_bounds(const StreamHost &S, int32_t n_vidx, std::string &why)
{
    if (S.esize != 4 && S.esize != 8) { why = "element size"; return false; }
    if (S.vix.size() != S.sub.size() * ((size_t)S.Kcap + S.Ccap + 1)) { why = "emission index table size"; return false; }
    for (const SubDesc &sd : S.sub) {
        if (sd.wave_ptr0 < 0 || (size_t)sd.wave_ptr0 + S.nw > S.waves.size()) { why = "wave table range"; return false; }
        if (sd.K > S.Kcap || sd.n_slot > S.Ccap) { why = "index space"; return false; }
        if (sd.clone0 < 0 || sd.n_cdesc < 0 || (size_t)sd.clone0 + (size_t)sd.n_cdesc > S.clones.size()) { why = "clone range"; return false; }
        if (sd.zero0 < 0 || sd.n_zero < 0 || (size_t)sd.zero0 + (size_t)sd.n_zero > S.zero_rows.size()) { why = "zero-row range"; return false; }
        for (int32_t c = 0; c < sd.n_cdesc; ++c) {
            const CloneDesc &cd = S.clones[(size_t)sd.clone0 + c];
            if (cd.state < 0 || cd.state >= sd.K || cd.first < 0 || cd.count < 1 || cd.first + cd.count > sd.n_slot) { why = "clone entry"; return false; }
        }
        for (int32_t z = 0; z < sd.n_zero; ++z)
            if (S.zero_rows[(size_t)sd.zero0 + z] < 0 || S.zero_rows[(size_t)sd.zero0 + z] >= sd.K) { why = "zero row"; return false; }
        for (int wv = 0; wv < S.nw; ++wv) {
            const WaveDesc &wd = S.waves[(size_t)sd.wave_ptr0 + wv];
            if (wd.n_iter < 0 || wd.n_iter > 2 * kWave || wd.flag_base < 0 ||
                (size_t)wd.flag_base + 2 + wd.n_iter > S.flagwords.size()) {
                why = "flag range";
                return false;
            }
            const size_t n_batches = wave_batches(wd);
            if (wd.arc_base < 0 || (size_t)wd.arc_base + n_batches * kBatchEntries > S.arcs.size()) {
                why = "stream range";
                return false;
            }
            for (size_t bt = 0; bt < n_batches; ++bt) {
                const uint32_t f = batch_flags(S, wd, bt);
                if (((f >> kFlagLgShift) & 7u) > 6u) { why = "lanes per row"; return false; }
                const bool dual = (f & kFlagDual) != 0, quad = (f & kFlagQuad) != 0;
                if ((dual || quad) && (bt >= (size_t)kMaxStacked || !(f & kFlagInfo) || (dual && quad) || ((f >> kFlagLgShift) & 7u) ||
                                       (f & kFlagSkip))) {
                    why = "stacked batch";
                    return false;
                }
                for (int r = 0; r < kBatchRows; ++r)
                    for (int lane = 0; lane < kWave; ++lane) {
                        const Arc &a = S.arcs[(size_t)wd.arc_base + entry_at(bt, r, lane)];
                        // rows that end a part carry a target
                        const bool closing = (f & kFlagInfo) && (r == kBatchRows - 1 || quad || (dual && r % 2 == 1));
                        const int32_t off = closing ? (int32_t)((uint32_t)a.src & 0xffffu) : a.src;
                        const int32_t src = off / S.esize;
                        if (off < 0 || off % S.esize || (src >= sd.K && (src < S.Kcap || src >= S.Kcap + sd.n_slot))) {
                            why = "arc source";
                            return false;
                        }
                        if (!(a.w <= 0.0f) && !(a.w > 0.0f)) { why = "NaN weight"; return false; }
                        if (closing) {
                            const int32_t t = (int32_t)((uint32_t)a.src >> 16);
                            const bool state = t < sd.K, slot = t >= S.Kcap && t < S.Kcap + sd.n_slot;
                            const bool dump = t == S.Kcap + S.Ccap;
                            if (!state && !slot && !dump) { why = "row target"; return false; }
                            const int32_t v = S.vix[(size_t)(&sd - S.sub.data()) * ((size_t)S.Kcap + S.Ccap + 1) + (size_t)t];
                            if (v != S.Ecap && v >= (n_vidx < 0 ? sd.K : n_vidx)) { why = "emission index"; return false; }
                            if (dump && v != S.Ecap) { why = "emission on the dump slot"; return false; }
                        }
                    }
            }
        }
    }
    return true;
}

// The streams of sub-graph `sub` interpreted on the host in double precision as the kernel
// does (lanes, groups of lanes, clones): y[state] for every state, before emission and offset
// are applied; x holds one value per state.
bool stream_apply_host(const StreamHost &S, int32_t sub, const double *x, double *y, const std::vector<Arc> *lin, std::string &why)
{
    const SubDesc &sd = S.sub[(size_t)sub];
    // the vector the rows gather from: a cloned state's value sits in the state itself, its clones hold zero
    std::vector<double> xe(x, x + sd.K);
    xe.resize((size_t)sd.K + (size_t)sd.n_slot, -INFINITY);
    std::vector<double> ye((size_t)sd.K + (size_t)sd.n_slot, -INFINITY);
    auto lse = [](const std::vector<double> &t) {
        double m = -INFINITY, acc = 0.0;
        for (double v : t) m = std::max(m, v);
        if (m == -INFINITY) return m;
        for (double v : t) acc += std::exp2(v - m);
        return m + std::log2(acc);
    };
    for (int wv = 0; wv < S.nw; ++wv) {
        const WaveDesc &wd = S.waves[(size_t)sd.wave_ptr0 + wv];
        const size_t n_batches = wave_batches(wd);
        std::vector<std::vector<double>> terms(kWave);   // running (+)-sum of every lane, kept as its terms
        for (size_t bt = 0; bt < n_batches; ++bt) {
            const uint32_t f = batch_flags(S, wd, bt);
            if (f & kFlagSkip) continue;
            if (f & (kFlagDual | kFlagQuad)) {   // stacked slices: every part of a lane is a row of its own, closed here
                const int rows_per = (f & kFlagQuad) ? 1 : 2;
                for (int lane = 0; lane < kWave; ++lane)
                    for (int part = 0; part < kBatchRows / rows_per; ++part) {
                        std::vector<double> tm;
                        int32_t t = 0;
                        for (int j = 0; j < rows_per; ++j) {
                            const Arc &a = S.arcs[(size_t)wd.arc_base + entry_at(bt, part * rows_per + j, lane)];
                            const bool last = j == rows_per - 1;
                            const int32_t src = (last ? (int32_t)((uint32_t)a.src & 0xffffu) : a.src) / S.esize;
                            tm.push_back((double)a.w + xe[(size_t)(src < sd.K ? src : sd.K + (src - S.Kcap))]);
                            if (last) t = (int32_t)((uint32_t)a.src >> 16);
                        }
                        if (t < sd.K) ye[(size_t)t] = lse(tm);
                        else if (t < S.Kcap + sd.n_slot) ye[(size_t)sd.K + (size_t)(t - S.Kcap)] = lse(tm);
                    }
                continue;
            }
            const int g = 1 << ((f >> kFlagLgShift) & 7u);
            const std::vector<Arc> &arcs = lin ? *lin : S.arcs;
            const int32_t dump = S.Kcap + S.Ccap;
            for (int r = 0; r < kBatchRows; ++r)
                for (int lane = 0; lane < kWave; ++lane) {
                    const Arc &a = arcs[(size_t)wd.arc_base + entry_at(bt, r, lane)];
                    const bool closing = r == kBatchRows - 1 && (f & kFlagInfo);
                    const int32_t src = (closing ? (int32_t)((uint32_t)a.src & 0xffffu) : a.src) / S.esize;
                    if (lin) {
                        // weights as 2^w: an entry of weight 0 must gather the dump slot (zero-bar), or the
                        // kernel's running maximum, which is over the gathered values alone, could exceed every term
                        if (a.w == 0.0f && src != dump) { why = "an entry of weight 0 gathers a state"; return false; }
                        if (a.w != 0.0f && src == dump) { why = "a weighted entry gathers the dump slot"; return false; }
                        const double xv = src == dump ? -INFINITY : xe[(size_t)(src < sd.K ? src : sd.K + (src - S.Kcap))];
                        terms[lane].push_back((a.w == 0.0f ? -INFINITY : std::log2((double)a.w)) + xv);
                        continue;
                    }
                    terms[lane].push_back((double)a.w + xe[(size_t)(src < sd.K ? src : sd.K + (src - S.Kcap))]);
                }
            if (f & kFlagInfo) {
                for (int lane = 0; lane < kWave; lane += g) {   // the row's lanes are complete
                    std::vector<double> all;
                    for (int t = 0; t < g; ++t) all.insert(all.end(), terms[lane + t].begin(), terms[lane + t].end());
                    for (int t = 0; t < g; ++t) terms[lane + t].assign(1, lse(all));   // every lane of the row holds the total
                }
                for (int lane = 0; lane < kWave; ++lane) {
                    const Arc &a = arcs[(size_t)wd.arc_base + entry_at(bt, kBatchRows - 1, lane)];
                    const int32_t t = (int32_t)((uint32_t)a.src >> 16);
                    if (lin && t == dump && terms[lane][0] != -INFINITY) { why = "a row's total goes to the dump slot"; return false; }
                    if (t < sd.K) ye[(size_t)t] = terms[lane][0];
                    else if (t < S.Kcap + sd.n_slot) ye[(size_t)sd.K + (size_t)(t - S.Kcap)] = terms[lane][0];
                    terms[lane].clear();
                }
            }
        }
    }
    for (int32_t c = 0; c < sd.n_cdesc; ++c) {   // a cloned state is the (+)-sum of its clones
        const CloneDesc &cd = S.clones[(size_t)sd.clone0 + c];
        std::vector<double> all{ye[(size_t)cd.state]};
        for (int32_t i = 0; i < cd.count; ++i) all.push_back(ye[(size_t)sd.K + (size_t)cd.first + i]);
        ye[(size_t)cd.state] = lse(all);
    }
    for (int32_t k = 0; k < sd.K; ++k) y[k] = ye[(size_t)k];
    return true;
}

bool stream_linear_weights(const StreamHost &S, std::vector<Arc> &out)
{
    out = S.arcs;
    const uint32_t dump_off = (uint32_t)(S.Kcap + S.Ccap) * (uint32_t)S.esize;
    const size_t per_batch = (size_t)kBatchEntries;
    for (const WaveDesc &wd : S.waves) {
        bool live[kWave] = {};   // the lane has had an arc of finite weight since its last row ended
        for (size_t q = 0; q < wave_batches(wd); ++q) {
            if (batch_flags(S, wd, q) & (kFlagDual | kFlagQuad)) continue;   // stacked batches add in the exponent as before
            Arc *a = out.data() + (size_t)wd.arc_base + q * per_batch;
            // A row spread over 2^lg lanes ends with its total in every lane of the group; the plan lets only the
            // group's first lane write it and sends the others to the dump slot.  Here the dump slot must keep
            // zero-bar, so the other lanes write the same value to the same state instead.
            const uint32_t fl = batch_flags(S, wd, q);
            const int lg = (int)((fl >> kFlagLgShift) & 7u);
            if ((fl & kFlagInfo) && lg > 0) {
                const uint32_t dump = (uint32_t)(S.Kcap + S.Ccap);
                for (int lane = 0; lane < kWave; ++lane) {
                    Arc &e = a[entry_at(0, kBatchRows - 1, lane)];
                    const Arc &first = a[entry_at(0, kBatchRows - 1, lane & ~((1 << lg) - 1))];
                    if (((uint32_t)e.src >> 16) == dump)
                        e.src = (int32_t)(((uint32_t)e.src & 0xffffu) | ((uint32_t)first.src & 0xffff0000u));
                }
            }
            for (int lane = 0; lane < kWave; ++lane)
                for (int r = 0; r < kBatchRows; ++r) {
                    Arc &e = a[entry_at(0, r, lane)];
                    if (e.w == -INFINITY) {
                        e.src = (int32_t)(((uint32_t)e.src & 0xffff0000u) | dump_off);
                        e.w = 0.0f;
                    } else {
                        if (!(e.w >= -kLinearSpan && e.w <= kLinearSpan)) return false;
                        e.w = exp2f(e.w);
                        live[lane] = true;
                    }
                }
            if (fl & kFlagInfo)   // rows end here: nothing but zero-bar may go to the dump slot
                for (int lane = 0; lane < kWave; ++lane) {
                    if (live[lane] && ((uint32_t)a[entry_at(0, kBatchRows - 1, lane)].src >> 16) == (uint32_t)(S.Kcap + S.Ccap)) return false;
                    live[lane] = false;
                }
        }
    }
    return true;
}

}  // namespace fb
