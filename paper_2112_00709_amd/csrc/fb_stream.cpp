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

}  // namespace

bool stream_from_sell(const SellHost &S, StreamHost &out, std::string &why)
{
    out.nw = S.nw;
    out.max_part = S.max_part;
    for (const SubDesc &ssd : S.sub) {
        if (ssd.K >= (int32_t)kOutPartial || ssd.n_part >= (int32_t)kOutPartial) {
            why = "more than 32767 states or partial slots in one (sub-)graph";
            return false;
        }
        SubDesc sd = ssd;
        sd.wave_ptr0 = (int32_t)out.waves.size();
        for (int wv = 0; wv < S.nw; ++wv) {
            WaveDesc wd{};
            wd.arc_base = (int64_t)out.arcs.size();
            std::vector<uint8_t> flags;   // one per batch
            for (int32_t l = 0; l < ssd.n_levels; ++l) {
                const int32_t s0 = S.wave_ptr[(size_t)ssd.wave_ptr0 + l * S.nw + wv];
                const int32_t s1 = S.wave_ptr[(size_t)ssd.wave_ptr0 + l * S.nw + wv + 1];
                std::vector<uint8_t> row_is_info;
                for (int32_t s = s0; s < s1; ++s) {
                    const int32_t trip = S.slice_trip[s];
                    for (int32_t it = 0; it < trip; ++it) {
                        for (int lane = 0; lane < kWave; ++lane)
                            out.arcs.push_back(S.arcs[(size_t)S.slice_arc[s] + (size_t)it * kWave + lane]);
                        row_is_info.push_back(0);
                    }
                    for (int lane = 0; lane < kWave; ++lane) {
                        const int32_t o = S.row_out[(size_t)s * kWave + lane], v = S.row_vidx[(size_t)s * kWave + lane];
                        if (v < 0 || v > 0xffff) { why = "emission index beyond 16 bits"; return false; }
                        const uint32_t o16 = o >= 0 ? (uint32_t)o : o == -1 ? kOutIdle : (kOutPartial | (uint32_t)(-2 - o));
                        out.arcs.push_back(Arc{0, bits_to_float(o16 | ((uint32_t)v << 16))});
                    }
                    row_is_info.push_back(1);
                }
                // pad the level to whole batches with info rows that go nowhere; a wave without
                // work at this level still gets one (skipped) batch to carry the barrier flag
                const bool idle = row_is_info.empty();
                while (row_is_info.empty() || row_is_info.size() % kBatchRows) {
                    for (int lane = 0; lane < kWave; ++lane) out.arcs.push_back(Arc{0, bits_to_float(kOutIdle)});
                    row_is_info.push_back(1);
                }
                for (size_t r = 0; r < row_is_info.size(); r += kBatchRows) {
                    uint8_t f = idle ? (uint8_t)kFlagSkip : 0;
                    for (int j = 0; j < kBatchRows; ++j)
                        if (row_is_info[r + j]) f |= (uint8_t)(1u << j);
                    flags.push_back(f);
                }
                if (l + 1 < ssd.n_levels) flags.back() |= (uint8_t)kFlagLevelEnd;
            }
            while (flags.empty() || flags.size() % kRing) {   // whole unrolled iterations
                for (int e = 0; e < kBatchEntries; ++e) out.arcs.push_back(Arc{0, bits_to_float(kOutIdle)});
                flags.push_back((uint8_t)(kFlagSkip | kFlagInfoMask));
            }
            if (flags.size() / kRing > 2 * kWave) {
                why = "more than " + std::to_string(2 * kWave * kRing * kBatchRows * kWave) + " arcs per wave and time step";
                return false;
            }
            wd.n_iter = (int32_t)(flags.size() / kRing);
            wd.flag_base = (int32_t)out.flagwords.size();
            for (size_t i = 0; i < flags.size(); i += kRing) {
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
        int32_t barriers = -1;
        for (int wv = 0; wv < S.nw; ++wv) {
            const WaveDesc &wd = S.waves[(size_t)sd.wave_ptr0 + wv];
            if (wd.n_iter < 1 || wd.n_iter > 2 * kWave || wd.flag_base < 0 || (size_t)wd.flag_base + wd.n_iter > S.flagwords.size()) {
                why = "flag range";
                return false;
            }
            const size_t n_batches = (size_t)wd.n_iter * kRing;
            if (wd.arc_base < 0 || (size_t)wd.arc_base + n_batches * kBatchEntries > S.arcs.size()) {
                why = "stream range";
                return false;
            }
            int32_t level = 0, nbar = 0;
            for (size_t bt = 0; bt < n_batches; ++bt) {
                const uint32_t f = (S.flagwords[(size_t)wd.flag_base + bt / kRing] >> (8 * (bt % kRing))) & 0xff;
                for (int r = 0; r < kBatchRows; ++r)
                    for (int lane = 0; lane < kWave; ++lane) {
                        const Arc &a = S.arcs[(size_t)wd.arc_base + (bt * kBatchRows + r) * kWave + lane];
                        // the gather is issued for info rows too: src must be safe in every row
                        const int32_t lim = level == 0 ? sd.K : std::max(sd.n_part, 1);
                        if (a.src < 0 || a.src >= lim) { why = "arc source"; return false; }
                        if ((f >> r) & 1) {
                            const uint32_t u = float_to_bits(a.w), o16 = u & 0xffff, v = u >> 16;
                            if (o16 != kOutIdle) {
                                if (o16 & kOutPartial) {
                                    if ((int32_t)(o16 & 0x7fff) >= sd.n_part) { why = "partial slot"; return false; }
                                } else if ((int32_t)o16 >= sd.K) { why = "row target"; return false; }
                                if ((int32_t)v >= (n_vidx < 0 ? sd.K : n_vidx)) { why = "emission index"; return false; }
                            }
                        }
                    }
                if (f & kFlagLevelEnd) { ++level; ++nbar; }
            }
            if (barriers >= 0 && nbar != barriers) { why = "waves disagree on the number of barriers"; return false; }
            barriers = nbar;
            if (nbar != std::max(sd.n_levels, 1) - 1) { why = "barrier count"; return false; }
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
            const size_t n_batches = (size_t)wd.n_iter * kRing;
            std::vector<std::vector<double>> terms(kWave);   // running (+)-sum of every lane, kept as its terms
            while (at[wv] < n_batches) {
                const size_t bt = at[wv]++;
                const uint32_t f = (S.flagwords[(size_t)wd.flag_base + bt / kRing] >> (8 * (bt % kRing))) & 0xff;
                if (!(f & kFlagSkip))
                    for (int r = 0; r < kBatchRows; ++r)
                        for (int lane = 0; lane < kWave; ++lane) {
                            const Arc &a = S.arcs[(size_t)wd.arc_base + (bt * kBatchRows + r) * kWave + lane];
                            if (!((f >> r) & 1)) {
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
                            const uint32_t o16 = float_to_bits(a.w) & 0xffff;
                            if (o16 == kOutIdle) continue;
                            if (o16 & kOutPartial) writes.emplace_back((int32_t)(o16 & 0x7fff), acc);
                            else y[o16] = acc;
                        }
                if (f & kFlagLevelEnd) break;
            }
        }
        for (auto &wr : writes) part[(size_t)wr.first] = wr.second;
    }
}

}  // namespace fb
