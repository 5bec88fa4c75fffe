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

bool stream_from_sell(const SellHost &S, int32_t Kcap, int32_t Ecap, StreamHost &out, std::string &why)
{
    out.nw = S.nw;
    out.Kcap = Kcap;
    out.Pcap = S.max_part;
    out.Ecap = Ecap;
    if ((int64_t)Kcap + S.max_part + 1 > 0xffff || Ecap + 1 > 0xffff) {
        why = "states plus partial slots, or emission entries, beyond 16 bits";
        return false;
    }
    const uint32_t idle_info = (uint32_t)(Kcap + S.max_part) | ((uint32_t)Ecap << 16);
    const Arc pad_arc{0, -INFINITY};
    for (const SubDesc &ssd : S.sub) {
        SubDesc sd = ssd;
        sd.wave_ptr0 = (int32_t)out.waves.size();
        for (int wv = 0; wv < S.nw; ++wv) {
            WaveDesc wd{};
            wd.arc_base = (int64_t)out.arcs.size();
            std::vector<uint8_t> flags;   // one per batch
            std::vector<Arc> lin;         // the wave's rows in order, 64 entries each
            auto pad_batch = [&](uint8_t f) {   // three zero-weight arcs and an info row that goes to the dump slot
                for (int e = 0; e < (kBatchRows - 1) * kWave; ++e) lin.push_back(pad_arc);
                for (int lane = 0; lane < kWave; ++lane) lin.push_back(Arc{0, bits_to_float(idle_info)});
                flags.push_back((uint8_t)(f | kFlagInfo | kFlagSkip));
            };
            for (int32_t l = 0; l < ssd.n_levels; ++l) {
                const int32_t s0 = S.wave_ptr[(size_t)ssd.wave_ptr0 + l * S.nw + wv];
                const int32_t s1 = S.wave_ptr[(size_t)ssd.wave_ptr0 + l * S.nw + wv + 1];
                const size_t first_flag = flags.size();
                for (int32_t s = s0; s < s1; ++s) {
                    const int32_t trip = S.slice_trip[s];
                    int32_t rows = 0;
                    for (int32_t it = 0; it < trip; ++it, ++rows)
                        for (int lane = 0; lane < kWave; ++lane)
                            lin.push_back(S.arcs[(size_t)S.slice_arc[s] + (size_t)it * kWave + lane]);
                    for (; rows % kBatchRows != kBatchRows - 1; ++rows)   // the info row closes a batch
                        for (int lane = 0; lane < kWave; ++lane) lin.push_back(pad_arc);
                    for (int lane = 0; lane < kWave; ++lane) {
                        const int32_t o = S.row_out[(size_t)s * kWave + lane], v = S.row_vidx[(size_t)s * kWave + lane];
                        uint32_t info = idle_info;
                        if (o >= 0) info = (uint32_t)o | ((uint32_t)v << 16);
                        else if (o < -1) info = (uint32_t)(Kcap + (-2 - o)) | ((uint32_t)Ecap << 16);   // partial: no emission
                        lin.push_back(Arc{0, bits_to_float(info)});
                    }
                    ++rows;
                    for (int32_t bt = 0; bt < rows / kBatchRows; ++bt)
                        flags.push_back(bt + 1 == rows / kBatchRows ? (uint8_t)kFlagInfo : (uint8_t)0);
                }
                if (flags.size() == first_flag) pad_batch(0);   // a wave without work here still carries the barrier
                if (l + 1 < ssd.n_levels) flags.back() |= (uint8_t)kFlagLevelEnd;
            }
            while (flags.size() < (size_t)kResident || (flags.size() - kResident) % kRing) pad_batch(0);   // whole iterations
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
    for (const SubDesc &sd : S.sub) {
        if (sd.wave_ptr0 < 0 || (size_t)sd.wave_ptr0 + S.nw > S.waves.size()) { why = "wave table range"; return false; }
        if (sd.K > S.Kcap || sd.n_part > S.Pcap) { why = "index space"; return false; }
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
            int32_t level = 0;
            for (size_t bt = 0; bt < n_batches; ++bt) {
                const uint32_t f = batch_flags(S, wd, bt);
                for (int r = 0; r < kBatchRows; ++r)
                    for (int lane = 0; lane < kWave; ++lane) {
                        const Arc &a = S.arcs[(size_t)wd.arc_base + entry_at(bt, r, lane)];
                        // every row is gathered, info rows included: src must always be safe
                        const int32_t lim = level == 0 ? sd.K : std::max(sd.n_part, 1);
                        if (a.src < 0 || a.src >= lim) { why = "arc source"; return false; }
                        if (r == kBatchRows - 1 && (f & kFlagInfo)) {
                            const uint32_t u = float_to_bits(a.w);
                            const int32_t t = (int32_t)(u & 0xffff), v = (int32_t)(u >> 16);
                            const bool state = t < sd.K, slot = t >= S.Kcap && t < S.Kcap + sd.n_part;
                            const bool dump = t == S.Kcap + S.Pcap;
                            if (!state && !slot && !dump) { why = "row target"; return false; }
                            if (v != S.Ecap && v >= (n_vidx < 0 ? sd.K : n_vidx)) { why = "emission index"; return false; }
                            if (!state && v != S.Ecap) { why = "emission on a partial row"; return false; }
                        } else if (!(a.w <= 0.0f) && !(a.w > 0.0f)) {
                            why = "NaN weight";
                            return false;
                        }
                    }
                if (f & kFlagLevelEnd) ++level;
            }
            if (level != std::max(sd.n_levels, 1) - 1) { why = "barrier count"; return false; }
            if (batch_flags(S, wd, n_batches - 1) & kFlagLevelEnd) { why = "barrier on the last batch"; return false; }
        }
    }
    return true;
}

// The streams of sub-graph `sub` interpreted on the host in double precision,
// level by level as the kernel does between barriers: y[state] for every row that
// targets a state (before emission and offset are applied).
void stream_apply_host(const StreamHost &S, int32_t sub, const double *x, double *y)
{
    const SubDesc &sd = S.sub[(size_t)sub];
    std::vector<double> part((size_t)std::max(sd.n_part, 1), 0.0);
    std::vector<size_t> at((size_t)S.nw, 0);   // next batch of every wave
    for (int32_t l = 0; l < std::max(sd.n_levels, 1); ++l) {
        const double *v = l == 0 ? x : part.data();
        std::vector<std::pair<int32_t, double>> writes;
        for (int wv = 0; wv < S.nw; ++wv) {
            const WaveDesc &wd = S.waves[(size_t)sd.wave_ptr0 + wv];
            const size_t n_batches = wave_batches(wd);
            std::vector<std::vector<double>> terms(kWave);   // running (+)-sum of every lane, kept as its terms
            while (at[wv] < n_batches) {
                const size_t bt = at[wv]++;
                const uint32_t f = batch_flags(S, wd, bt);
                if (!(f & kFlagSkip))
                    for (int r = 0; r < kBatchRows; ++r)
                        for (int lane = 0; lane < kWave; ++lane) {
                            const Arc &a = S.arcs[(size_t)wd.arc_base + entry_at(bt, r, lane)];
                            if (!(r == kBatchRows - 1 && (f & kFlagInfo))) {
                                terms[lane].push_back((double)a.w + v[a.src]);
                                continue;
                            }
                            double m = -INFINITY, acc = 0.0;
                            for (double t : terms[lane]) m = std::max(m, t);
                            if (m == -INFINITY) acc = -INFINITY;
                            else {
                                for (double t : terms[lane]) acc += std::exp2(t - m);
                                acc = m + std::log2(acc);
                            }
                            terms[lane].clear();
                            const int32_t t = (int32_t)(float_to_bits(a.w) & 0xffff);
                            if (t < sd.K) y[t] = acc;
                            else if (t < S.Kcap + S.Pcap) writes.emplace_back(t - S.Kcap, acc);
                        }
                if (f & kFlagLevelEnd) break;
            }
        }
        for (auto &wr : writes) part[(size_t)wr.first] = wr.second;
    }
}

}  // namespace fb
