// Graph handle: validation, the graph-layout step (stable sorts by destination,
// by source and by pdf), the kernel schedules built from those layouts, upload.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cstdlib>
#include <cmath>
#include <cstring>
#include <new>
#include <numeric>

#include "fb_internal.h"

namespace fb {

static thread_local std::string g_err;

void set_error(const std::string &msg) { g_err = msg; }

int fail(int code, const std::string &msg)
{
    g_err = msg;
    return code;
}

namespace {

constexpr double kLog2e = 1.4426950408889634074;

// ptr/perm of the stable ascending order of keys in [0, n_keys): counting sort,
// scanning the input left to right, so ties keep their original order.
void stable_group(const int32_t *keys, int64_t n, int32_t n_keys, std::vector<int32_t> &ptr, std::vector<int32_t> &perm)
{
    ptr.assign((size_t)n_keys + 1, 0);
    for (int64_t i = 0; i < n; ++i) ++ptr[(size_t)keys[i] + 1];
    for (int32_t k = 0; k < n_keys; ++k) ptr[k + 1] += ptr[k];
    perm.resize((size_t)n);
    std::vector<int32_t> at(ptr.begin(), ptr.end() - 1);
    for (int64_t i = 0; i < n; ++i) perm[(size_t)at[keys[i]]++] = (int32_t)i;
}

float to_log2(float x) { return (float)((double)x * kLog2e); }   // -inf stays -inf

// rows [0, K) of a CSR-like matrix with parallel entries (same row and column) combined: (+) of the log
// semiring (log2 of the sum of the powers of two, in double) or, tropical, their maximum.  Columns come out
// in ascending order inside a row.  Returns whether anything was combined.
bool merge_parallel(int32_t K, const std::vector<int64_t> &ptr, const std::vector<int32_t> &col, const std::vector<float> &w,
                    bool tropical, std::vector<int64_t> &mptr, std::vector<int32_t> &mcol, std::vector<float> &mw)
{
    mptr.assign((size_t)K + 1, 0);
    mcol.clear();
    mw.clear();
    bool any = false;
    std::vector<std::pair<int32_t, float>> row;
    for (int32_t r = 0; r < K; ++r) {
        row.clear();
        for (int64_t e = ptr[r]; e < ptr[r + 1]; ++e) row.emplace_back(col[(size_t)e], w[(size_t)e]);
        std::stable_sort(row.begin(), row.end(), [](const std::pair<int32_t, float> &a, const std::pair<int32_t, float> &b) {
            return a.first < b.first;
        });
        for (size_t i = 0; i < row.size();) {
            size_t j = i + 1;
            double m = row[i].second;
            while (j < row.size() && row[j].first == row[i].first) m = std::max(m, (double)row[j++].second);
            double v = m;
            if (j > i + 1) {
                any = true;
                if (!tropical && m != -INFINITY) {
                    double s = 0.0;
                    for (size_t t = i; t < j; ++t) s += std::exp2((double)row[t].second - m);
                    v = m + std::log2(s);
                }
            }
            mcol.push_back(row[i].first);
            mw.push_back((float)v);
            i = j;
        }
        mptr[(size_t)r + 1] = (int64_t)mcol.size();
    }
    return any;
}

template <class T>
int upload(fb_graph *g, const std::vector<T> &h, const T **dev)
{
    *dev = nullptr;
    if (h.empty()) return FB_OK;
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, h.size() * sizeof(T));
    if (e != hipSuccess)
        return fail(e == hipErrorOutOfMemory ? FB_ENOMEM : FB_EHIP, std::string("hipMalloc: ") + hipGetErrorString(e));
    g->allocs.push_back(p);
    e = hipMemcpy(p, h.data(), h.size() * sizeof(T), hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail(FB_EHIP, std::string("hipMemcpy: ") + hipGetErrorString(e));
    *dev = (const T *)p;
    return FB_OK;
}

int upload_pdf(fb_graph *g, const PdfHost &h, PdfDev &d)
{
    int rc;
    if ((rc = upload(g, h.sub, &d.sub))) return rc;
    if ((rc = upload(g, h.row_pdf, &d.row_pdf))) return rc;
    if ((rc = upload(g, h.row_ptr, &d.row_ptr))) return rc;
    if ((rc = upload(g, h.pos, &d.pos))) return rc;
    return upload(g, h.states, &d.states);
}

// arcs: the list to upload in place of h.arcs (same length), or nullptr
int upload_stream(fb_graph *g, const StreamHost &h, StreamDev &d, const std::vector<Arc> *arcs = nullptr)
{
    int rc;
    if ((rc = upload(g, h.sub, &d.sub))) return rc;
    if ((rc = upload(g, h.waves, &d.waves))) return rc;
    if ((rc = upload(g, h.flagwords, &d.flagwords))) return rc;
    if ((rc = upload(g, h.vix, &d.vix))) return rc;
    if ((rc = upload(g, h.clones, &d.clones))) return rc;
    if ((rc = upload(g, h.zero_rows, &d.zero_rows))) return rc;
    return upload(g, arcs ? *arcs : h.arcs, &d.arcs);
}

}  // namespace

size_t recursion_lds_bytes(int32_t Kcap, int32_t Ccap, int32_t Ecap, bool backward, bool f64, bool shared, bool tropical,
                           int32_t xs_fixed)
{
    // carrier-typed: state buffers (states, clone slots, a dump slot) and reduction slots;
    // then three emission rows (float, plus a zero slot), for packed graphs a pdf id per state, the emission index table
    const size_t xs = xs_fixed ? (size_t)xs_fixed : (size_t)Kcap + (size_t)Ccap + 1;
    return (xs * (backward ? 4 : 2) + 4 * kNWShared + 2) * (f64 ? 8 : 4) + ((size_t)Ecap + 1) * 12 +
           (shared ? 0 : (size_t)Ecap * 4) + (tropical ? xs * 4 : 0) + ((xs + 1) & ~(size_t)1) * 2 +
           kLdsReserve;   // tropical: two rows of 16-bit back-pointers; always: the 16-bit emission index of every target
}

size_t posterior_lds_bytes(const PostParams &p)
{
    // reduction slots, log posteriors of a double-carrier graph, per-state values, the pdf row,
    // then every graph's states-by-pdf table in 16-bit entries
    size_t n = 64 + (size_t)p.Kcap64 * 8 + ((size_t)p.Kcap + (size_t)p.D) * 4;
    for (int i = 0; i < p.n_graph; ++i) n += ((size_t)p.g[i].Rcap * 2 + 1 + (size_t)p.g[i].Kcap + 3) / 2 * 4;
    return n + kLdsReserve;
}

}  // namespace fb

using namespace fb;

extern "C" {

const char *fb_last_error(void) { return g_err.c_str(); }

const char *fb_strerror(int code)
{
    switch (code) {
    case FB_OK: return "success";
    case FB_EINVAL: return "invalid argument";
    case FB_ENOMEM: return "out of memory";
    case FB_EHIP: return "HIP runtime error";
    case FB_EUNSUPPORTED: return "input exceeds a limit of the kernels";
    default: return "unknown error code";
    }
}

int fb_graph_linear_weights(const fb_graph *g) { return g ? (g->linear_p ? 2 : g->linear_w ? 1 : 0) : -1; }

int64_t fb_debug_linear_restarts(void) { return (int64_t)linear_restarts(); }

int fb_graph_plan_cycles(const fb_graph *g, int backward, int64_t *cycles, int64_t *cycles_floor)
{
    if (!g || !cycles || !cycles_floor) return fail(FB_EINVAL, "fb_graph_plan_cycles: NULL argument");
    if (!g->linear_p) return fail(FB_EUNSUPPORTED, "fb_graph_plan_cycles: this graph has no probability-domain plan");
    const PStreamHost &S = backward ? g->hp_bwd : g->hp_fwd;
    std::vector<double> x((size_t)S.K, 1.0), y((size_t)S.K, 0.0);
    std::string why;
    if (!pstream_apply_host(S, x.data(), y.data(), cycles, cycles_floor, why))
        return fail(FB_EHIP, "internal error: probability-domain plan (" + why + ")");
    return FB_OK;
}

int32_t fb_limits_max_states(int32_t D, int shared)
{
    if (D <= 0) return 0;
    // backward recursion: four state vectors, clone slots (allow K/8), three emission rows
    // (D entries for a shared graph, one per state for packed graphs)
    const double avail = (double)kLdsBytes - (double)kLdsReserve - (shared ? 12.0 * D : 0.0);
    const double per_state = 4.0 * (4.0 + 0.125 + (shared ? 0.0 : 4.0)) + 2.0 * 1.125;   // + the 16-bit emission index table
    const double k = avail / per_state;
    return k < 1 ? 0 : (int32_t)k;
}

int fb_check_lengths(const int32_t *lengths_host, int32_t B, int32_t N)
{
    if (!lengths_host || B <= 0 || N <= 0) return fail(FB_EINVAL, "fb_check_lengths: NULL lengths or B, N <= 0");
    for (int32_t b = 0; b < B; ++b)
        if (lengths_host[b] < 1 || lengths_host[b] > N)
            return fail(FB_EINVAL, "length of sequence " + std::to_string(b) + " = " + std::to_string(lengths_host[b]) +
                                       " is outside [1, " + std::to_string(N) + "]");
    return FB_OK;
}

int fb_graph_create(fb_graph **out, int32_t K, int64_t E, const int32_t *src, const int32_t *dst, const float *logw,
                    const int32_t *pdf, const float *init, const float *final_, int32_t D, int32_t n_seq,
                    const int32_t *state_off, uint32_t flags)
{
    if (!out) return fail(FB_EINVAL, "fb_graph_create: out is NULL");
    *out = nullptr;
    if (K <= 0 || E < 0 || D <= 0) return fail(FB_EINVAL, "fb_graph_create: K <= 0, E < 0 or D <= 0");
    if (E > INT32_MAX / 2) return fail(FB_EUNSUPPORTED, "fb_graph_create: more than 2^30 arcs");
    if (D > 0xffff) return fail(FB_EUNSUPPORTED, "fb_graph_create: more than 65535 pdfs");
    if ((E > 0 && (!src || !dst || !logw)) || !pdf || !init || !final_)
        return fail(FB_EINVAL, "fb_graph_create: NULL array");
    if ((flags & FB_GRAPH_WIDE_STATE) && (flags & FB_GRAPH_NARROW_STATE))
        return fail(FB_EINVAL, "fb_graph_create: FB_GRAPH_WIDE_STATE and FB_GRAPH_NARROW_STATE exclude each other");
    if (n_seq < 0 || (n_seq > 0) != (state_off != nullptr))
        return fail(FB_EINVAL, "fb_graph_create: n_seq and state_off must be given together");
    for (int64_t e = 0; e < E; ++e) {
        if (src[e] < 0 || src[e] >= K || dst[e] < 0 || dst[e] >= K)
            return fail(FB_EINVAL, "arc " + std::to_string(e) + " has an endpoint outside [0, K)");
        if (std::isnan(logw[e]) || logw[e] == INFINITY)
            return fail(FB_EINVAL, "arc " + std::to_string(e) + " has a NaN or +inf weight");
    }
    for (int32_t k = 0; k < K; ++k) {
        if (pdf[k] < 0 || pdf[k] >= D) return fail(FB_EINVAL, "pdf id of state " + std::to_string(k) + " outside [0, D)");
        if (std::isnan(init[k]) || init[k] == INFINITY || std::isnan(final_[k]) || final_[k] == INFINITY)
            return fail(FB_EINVAL, "init/final of state " + std::to_string(k) + " is NaN or +inf");
    }
    std::vector<int32_t> seq_of;   // packed: sequence of every state
    if (n_seq > 0) {
        if (state_off[0] != 0 || state_off[n_seq] != K) return fail(FB_EINVAL, "state_off must run from 0 to K");
        seq_of.resize((size_t)K);
        for (int32_t b = 0; b < n_seq; ++b) {
            if (state_off[b + 1] <= state_off[b]) return fail(FB_EINVAL, "state_off must increase (no empty graph)");
            if (state_off[b + 1] > K) return fail(FB_EINVAL, "state_off beyond K");
            for (int32_t k = state_off[b]; k < state_off[b + 1]; ++k) seq_of[(size_t)k] = b;
        }
        for (int64_t e = 0; e < E; ++e)
            if (seq_of[(size_t)src[e]] != seq_of[(size_t)dst[e]])
                return fail(FB_EINVAL, "arc " + std::to_string(e) + " joins two packed graphs");
    }

    fb_graph *g = new (std::nothrow) fb_graph;
    if (!g) return fail(FB_ENOMEM, "fb_graph_create: host allocation failed");
    int rc = FB_OK;
    try {
        g->K = K; g->E = E; g->D = D; g->n_seq = n_seq;
        g->host_only = (flags & FB_GRAPH_HOST_ONLY) != 0;
        if (n_seq > 0) g->state_off.assign(state_off, state_off + n_seq + 1);

        // ---- graph-layout step: integer work, weights only permuted
        HostLayout &L = g->lay;
        stable_group(dst, E, K, L.in_ptr, L.in_perm);
        stable_group(src, E, K, L.out_ptr, L.out_perm);
        stable_group(pdf, K, D, L.pdf_ptr, L.pdf_states);
        L.in_src.resize((size_t)E); L.in_w.resize((size_t)E); L.out_dst.resize((size_t)E); L.out_w.resize((size_t)E);
        for (int64_t i = 0; i < E; ++i) {
            L.in_src[(size_t)i] = src[L.in_perm[(size_t)i]];
            L.in_w[(size_t)i] = logw[L.in_perm[(size_t)i]];
            L.out_dst[(size_t)i] = dst[L.out_perm[(size_t)i]];
            L.out_w[(size_t)i] = logw[L.out_perm[(size_t)i]];
        }

        // ---- schedules
        const int32_t n_sub = n_seq > 0 ? n_seq : 1;
        int64_t max_sub_E = 0;
        for (int32_t s = 0; s < n_sub; ++s) {
            const int32_t k0 = n_seq > 0 ? state_off[s] : 0, k1 = n_seq > 0 ? state_off[s + 1] : K;
            g->max_sub_K = std::max(g->max_sub_K, k1 - k0);
            max_sub_E = std::max<int64_t>(max_sub_E, (int64_t)L.in_ptr[k1] - L.in_ptr[k0]);
        }
        g->nw = (max_sub_E >= 4096 || g->max_sub_K > 1024) ? kNWShared : kNWSmall;
        g->f64 = (flags & FB_GRAPH_WIDE_STATE) ? true : (flags & FB_GRAPH_NARROW_STATE) ? false : g->nw == kNWSmall;
        SellHost sell_fwd, sell_bwd, sell_trop;   // sliced plans of the recursions, flattened into streams below
        sell_fwd.nw = sell_bwd.nw = sell_trop.nw = g->nw - 1;   // the last wave of a workgroup moves data, the others walk arcs
        bool any_parallel = false;
        bool prob_ok = n_seq == 0;   // the plans of the probability-domain kernel could be built

        std::vector<int64_t> ptr;
        std::vector<int32_t> col, vid;
        std::vector<float> w;
        for (int32_t s = 0; s < n_sub; ++s) {
            const int32_t k0 = n_seq > 0 ? state_off[s] : 0, k1 = n_seq > 0 ? state_off[s + 1] : K, Ks = k1 - k0;
            vid.resize((size_t)Ks);
            for (int32_t k = 0; k < Ks; ++k) vid[k] = n_seq > 0 ? k : pdf[k0 + k];
            for (int dir = 0; dir < 2; ++dir) {
                const std::vector<int32_t> &p = dir ? L.out_ptr : L.in_ptr, &other = dir ? L.out_dst : L.in_src;
                const std::vector<float> &ww = dir ? L.out_w : L.in_w;
                ptr.assign((size_t)Ks + 1, 0);
                const int64_t e0 = p[k0], e1 = p[k1];
                col.resize((size_t)(e1 - e0)); w.resize((size_t)(e1 - e0));
                for (int32_t k = 0; k <= Ks; ++k) ptr[k] = (int64_t)p[k0 + k] - e0;
                for (int64_t e = e0; e < e1; ++e) {
                    col[(size_t)(e - e0)] = other[(size_t)e] - k0;
                    w[(size_t)(e - e0)] = to_log2(ww[(size_t)e]);
                }
                // The plans carry one arc per (row, column): parallel arcs are (+)-added here, once, in double
                // (the exported layout keeps them apart).  The two semirings add differently, so the best-path
                // plan is a plan of its own as soon as the graph has parallel arcs.
                std::vector<int64_t> mptr;
                std::vector<int32_t> mcol;
                std::vector<float> mw;
                const bool dup = merge_parallel(Ks, ptr, col, w, false, mptr, mcol, mw);
                sell_append(dir ? sell_bwd : sell_fwd, k0, Ks, mptr.data(), mcol.data(), mw.data(), vid.data());
                // large shared graphs with float vectors: also the plan of the probability-domain kernel
                if (prob_ok && g->nw == kNWShared && !g->f64 && D <= 64 * kWave - 4) {   // (one mask bit per pdf in 64 x 64 bits, the row and its end marker in 1024 pieces)
                    std::string why;
                    PStreamHost &ps = dir ? g->hp_bwd : g->hp_fwd;
                    prob_ok = pstream_build(Ks, mptr.data(), mcol.data(), mw.data(), vid.data(), D, ps, why) &&
                              pstream_in_bounds(ps, D, why);
                } else {
                    prob_ok = false;
                }
                if (dir == 0) {
                    any_parallel = any_parallel || dup;
                    merge_parallel(Ks, ptr, col, w, true, mptr, mcol, mw);
                    sell_append(sell_trop, k0, Ks, mptr.data(), mcol.data(), mw.data(), vid.data());
                }
            }
            // states grouped by pdf: one row per pdf (every pdf for a shared graph, the pdfs the
            // sub-graph uses for packed graphs), states in ascending order inside a row
            PdfHost &PH = g->h_pdf;
            PdfSub ps{};
            ps.k0 = k0; ps.K = Ks;
            ps.row0 = (int32_t)PH.row_pdf.size(); ps.ptr0 = (int32_t)PH.row_ptr.size(); ps.st0 = (int32_t)PH.states.size();
            if (n_seq == 0) {
                for (int32_t d = 0; d < D; ++d) {
                    PH.row_pdf.push_back((uint16_t)d);
                    PH.row_ptr.push_back((uint16_t)L.pdf_ptr[d]);
                }
                PH.row_ptr.push_back((uint16_t)Ks);
                for (int32_t i = 0; i < Ks; ++i) PH.states.push_back((uint16_t)L.pdf_states[(size_t)i]);
                // padded to a multiple of 4 entries that point behind the states (read 4 at a time)
                PH.pos.assign((size_t)((Ks + 3) & ~3), (uint16_t)0);
                for (int32_t i = 0; i < Ks; ++i) PH.pos[(size_t)L.pdf_states[(size_t)i]] = (uint16_t)i;
                for (int32_t i = Ks; i < ((Ks + 3) & ~3); ++i) PH.pos[(size_t)i] = (uint16_t)i;
                ps.n_rows = D;
            } else {
                std::vector<int32_t> order((size_t)Ks);
                std::iota(order.begin(), order.end(), 0);
                std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return pdf[k0 + a] < pdf[k0 + b]; });
                for (size_t i = 0; i < order.size(); ++i) {
                    if (i == 0 || pdf[k0 + order[i]] != pdf[k0 + order[i - 1]]) {
                        PH.row_pdf.push_back((uint16_t)pdf[k0 + order[i]]);
                        PH.row_ptr.push_back((uint16_t)i);
                        ++ps.n_rows;
                    }
                    PH.states.push_back((uint16_t)order[i]);
                }
                PH.row_ptr.push_back((uint16_t)Ks);
            }
            PH.max_rows = std::max(PH.max_rows, ps.n_rows);
            PH.sub.push_back(ps);
        }
        std::vector<Arc> lin_fwd, lin_bwd;   // the arc lists with weights as 2^w, when the graph runs that instantiation
        {   // nothing a kernel will index may leave its array
            std::string why;
            const int32_t nv = n_seq > 0 ? -1 : D;
            if (!sell_in_bounds(sell_fwd, nv, why) || !sell_in_bounds(sell_bwd, nv, why))
                rc = fail(FB_EHIP, "internal error: schedule out of bounds (" + why + ")");
            else if (!stream_from_sell(sell_fwd, g->max_sub_K, n_seq > 0 ? g->max_sub_K : D, g->f64 ? 8 : 4, g->h_fwd, why) ||
                     !stream_from_sell(sell_bwd, g->max_sub_K, n_seq > 0 ? g->max_sub_K : D, g->f64 ? 8 : 4, g->h_bwd, why))
                rc = fail(FB_EUNSUPPORTED, "graph too large: " + why);
            else if (!stream_in_bounds(g->h_fwd, nv, why) || !stream_in_bounds(g->h_bwd, nv, why))
                rc = fail(FB_EHIP, "internal error: stream out of bounds (" + why + ")");
            // Large graphs with float vectors that fit the fixed-length buffers run the kernel instantiation that
            // takes weights as 2^w (one multiply-add per arc instead of an add before the exponential), unless a
            // weight is outside the range in which that is exact to rounding.  The best-path plan cannot share
            // such a stream.
            static const bool no_linear = getenv("FB_AMD_LINEAR") && getenv("FB_AMD_LINEAR")[0] == '0';   // (diagnostic switch)
            if (rc == FB_OK && !no_linear && !g->host_only && g->nw == kNWShared && !g->f64 &&
                g->max_sub_K + std::max(g->h_fwd.Ccap, g->h_bwd.Ccap) + 1 <= kXsFixed) {
                const int32_t Ecap1 = n_seq > 0 ? g->max_sub_K : D;
                g->linear_w = recursion_lds_bytes(g->max_sub_K, g->h_bwd.Ccap, Ecap1, true, false, n_seq == 0, false, kXsFixed) <= kLdsBytes &&
                              recursion_lds_bytes(g->max_sub_K, g->h_fwd.Ccap, Ecap1, false, false, n_seq == 0, false, kXsFixed) <= kLdsBytes &&
                              recursion_fixed_available() && stream_linear_weights(g->h_fwd, lin_fwd) &&
                              stream_linear_weights(g->h_bwd, lin_bwd);
            }
            // Large shared graphs with float vectors, at most 4096 pdfs and weights in range run their recursions in
            // the probability domain (one multiply-add per arc, one exponential per row; see linear_run); the
            // log form above stays on the device as what a sequence falls back to.
            static const bool no_prob = getenv("FB_AMD_PROBABILITY") && getenv("FB_AMD_PROBABILITY")[0] == '0';   // (diagnostic switch)
            if (rc == FB_OK && prob_ok && !no_prob && !g->host_only &&
                g->max_sub_K + std::max(g->h_fwd.Ccap, g->h_bwd.Ccap) + 1 <= kXsFixed &&
                std::max(recursion_lds_bytes(g->max_sub_K, g->h_bwd.Ccap, D, true, false, true, false, kXsFixed),
                         probability_lds_bytes(D, true)) <= kLdsBytes &&
                recursion_fixed_available()) {
                g->linear_p = true;
                g->linear_w = false;   // the log form it falls back to adds in the exponent
            }
            if (g->host_only && prob_ok) g->linear_p = true;   // (host-only handles keep the plans for fb_graph_schedule_apply_host)
            g->own_trop = any_parallel || g->linear_w;
            if (rc == FB_OK && g->own_trop) {
                if (!sell_in_bounds(sell_trop, nv, why))
                    rc = fail(FB_EHIP, "internal error: schedule out of bounds (" + why + ")");
                else if (!stream_from_sell(sell_trop, g->max_sub_K, n_seq > 0 ? g->max_sub_K : D, g->f64 ? 8 : 4, g->h_trop, why))
                    rc = fail(FB_EUNSUPPORTED, "graph too large: " + why);
                else if (!stream_in_bounds(g->h_trop, nv, why))
                    rc = fail(FB_EHIP, "internal error: stream out of bounds (" + why + ")");
            }
        }
        const int32_t Ccap = std::max(g->h_fwd.Ccap, g->h_bwd.Ccap);
        const int32_t Ecap = n_seq > 0 ? g->max_sub_K : D;
        if (rc == FB_OK && (recursion_lds_bytes(g->max_sub_K, g->h_fwd.Ccap, Ecap, false, g->f64, n_seq == 0) > kLdsBytes ||
            recursion_lds_bytes(g->max_sub_K, g->h_bwd.Ccap, Ecap, true, g->f64, n_seq == 0) > kLdsBytes)) {
            rc = fail(FB_EUNSUPPORTED, "graph too large: " + std::to_string(g->max_sub_K) + " states, " +
                                           std::to_string(Ccap) + " clone slots and " + std::to_string(Ecap) +
                                           " emission entries do not fit the on-chip memory of a compute unit");
        }

        // ---- upload
        if (rc == FB_OK && !g->host_only) {
            static_scratch_init();
            if (n_seq != 0) side_stream_init();
            std::vector<float> i2((size_t)K), f2((size_t)K);
            for (int32_t k = 0; k < K; ++k) { i2[k] = to_log2(init[k]); f2[k] = to_log2(final_[k]); }
            std::vector<int32_t> hp(pdf, pdf + K);
            const int32_t *dp = nullptr; const float *di = nullptr, *df = nullptr;
            if (!(rc = upload(g, hp, &dp)) && !(rc = upload(g, i2, &di)) && !(rc = upload(g, f2, &df)) &&
                !(rc = upload_stream(g, g->h_fwd, g->fwd, g->linear_w ? &lin_fwd : nullptr)) &&
                !(rc = upload_stream(g, g->h_bwd, g->bwd, g->linear_w ? &lin_bwd : nullptr)))
                rc = upload_pdf(g, g->h_pdf, g->pdfs);
            if (rc == FB_OK) {
                if (g->own_trop) rc = upload_stream(g, g->h_trop, g->trop);
                else g->trop = g->fwd;
            }
            if (rc == FB_OK && g->linear_p) {
                auto up = [&](const PStreamHost &h, PStreamDev &d) {
                    int r;
                    if ((r = upload(g, h.waves, &d.waves)) || (r = upload(g, h.units, &d.units)) ||
                        (r = upload(g, h.close_words, &d.close_words)) || (r = upload(g, h.clones, &d.clones)) ||
                        (r = upload(g, h.zero_rows, &d.zero_rows)))
                        return r;
                    d.n_clones = (int32_t)h.clones.size();
                    d.n_zero = (int32_t)h.zero_rows.size();
                    d.Ccap = h.Ccap;
                    d.bias = h.bias;
                    d.dim = h.dim;
                    return (int)FB_OK;
                };
                if (!(rc = up(g->hp_fwd, g->pfwd))) rc = up(g->hp_bwd, g->pbwd);
            }
            g->d_pdf = const_cast<int32_t *>(dp); g->d_init2 = const_cast<float *>(di); g->d_final2 = const_cast<float *>(df);
            if (rc == FB_OK && n_seq == 0) rc = leaky_prepare(g, init, final_);
        }
    } catch (const std::bad_alloc &) {
        rc = fail(FB_ENOMEM, "fb_graph_create: host allocation failed");
    }
    if (rc != FB_OK) {
        const std::string keep = fb_last_error();
        fb_graph_destroy(g);
        set_error(keep);
        return rc;
    }
    *out = g;
    return FB_OK;
}

int fb_graph_destroy(fb_graph *g)
{
    if (!g) return FB_OK;
    int rc = FB_OK;
    for (void *p : g->allocs)
        if (hipFree(p) != hipSuccess) rc = FB_EHIP;
    fb::leaky_release(g);
    delete g;
    return rc == FB_OK ? FB_OK : fail(FB_EHIP, "hipFree failed");
}

static const void *layout_array(const fb_graph *g, int which, int64_t *n)
{
    const HostLayout &L = g->lay;
    switch (which) {
    case FB_IN_PTR: *n = (int64_t)L.in_ptr.size(); return L.in_ptr.data();
    case FB_IN_SRC: *n = (int64_t)L.in_src.size(); return L.in_src.data();
    case FB_IN_W: *n = (int64_t)L.in_w.size(); return L.in_w.data();
    case FB_IN_PERM: *n = (int64_t)L.in_perm.size(); return L.in_perm.data();
    case FB_OUT_PTR: *n = (int64_t)L.out_ptr.size(); return L.out_ptr.data();
    case FB_OUT_DST: *n = (int64_t)L.out_dst.size(); return L.out_dst.data();
    case FB_OUT_W: *n = (int64_t)L.out_w.size(); return L.out_w.data();
    case FB_OUT_PERM: *n = (int64_t)L.out_perm.size(); return L.out_perm.data();
    case FB_PDF_PTR: *n = (int64_t)L.pdf_ptr.size(); return L.pdf_ptr.data();
    case FB_PDF_STATES: *n = (int64_t)L.pdf_states.size(); return L.pdf_states.data();
    default: *n = -1; return nullptr;
    }
}

int fb_graph_schedule_apply_host(const fb_graph *g, int which, int32_t sub, const double *x, double *y)
{
    if (!g || !x || !y) return fail(FB_EINVAL, "fb_graph_schedule_apply_host: NULL argument");
    if (which < 0 || which > 6 || sub < 0 || (size_t)sub >= g->h_pdf.sub.size())
        return fail(FB_EINVAL, "fb_graph_schedule_apply_host: unknown schedule or sub-graph");
    if (which >= 5) {   // the plans of the probability-domain kernel: ordinary arithmetic
        if (!g->linear_p) return fail(FB_EUNSUPPORTED, "fb_graph_schedule_apply_host: this graph has no probability-domain plan");
        std::string why;
        if (!pstream_apply_host(which == 5 ? g->hp_fwd : g->hp_bwd, x, y, nullptr, nullptr, why))
            return fail(FB_EHIP, "internal error: probability-domain plan (" + why + ")");
        return FB_OK;
    }
    if (which >= 3) {   // the forward / backward stream with weights as 2^w
        const StreamHost &S = which == 3 ? g->h_fwd : g->h_bwd;
        std::vector<Arc> lin;
        std::string why;
        if (!stream_linear_weights(S, lin)) return fail(FB_EUNSUPPORTED, "fb_graph_schedule_apply_host: the weights of this graph do not take the form 2^w");
        if (!stream_apply_host(S, sub, x, y, &lin, why)) return fail(FB_EHIP, "internal error: stream with weights as 2^w (" + why + ")");
        return FB_OK;
    }
    if (which == 2) {
        const PdfHost &PH = g->h_pdf;
        const PdfSub &ps = PH.sub[(size_t)sub];
        for (int32_t r = 0; r < ps.n_rows; ++r) {
            double acc = 0.0;
            for (int32_t i = PH.row_ptr[(size_t)ps.ptr0 + r]; i < PH.row_ptr[(size_t)ps.ptr0 + r + 1]; ++i)
                acc += x[PH.states[(size_t)ps.st0 + i]];
            y[PH.row_pdf[(size_t)ps.row0 + r]] = acc;
        }
    } else {
        std::string why;
        stream_apply_host(which == 0 ? g->h_fwd : g->h_bwd, sub, x, y, nullptr, why);
    }
    return FB_OK;
}

int64_t fb_graph_layout_size(const fb_graph *g, int which)
{
    if (!g) return fail(FB_EINVAL, "fb_graph_layout_size: NULL graph");
    int64_t n;
    layout_array(g, which, &n);
    if (n < 0) return fail(FB_EINVAL, "fb_graph_layout_size: unknown array");
    return n;
}

int fb_graph_layout(const fb_graph *g, int which, void *host_out, size_t bytes)
{
    if (!g || !host_out) return fail(FB_EINVAL, "fb_graph_layout: NULL argument");
    int64_t n;
    const void *p = layout_array(g, which, &n);
    if (n < 0) return fail(FB_EINVAL, "fb_graph_layout: unknown array");
    if (bytes != (size_t)n * 4) return fail(FB_EINVAL, "fb_graph_layout: bytes must be 4 * fb_graph_layout_size()");
    if (n) std::memcpy(host_out, p, bytes);
    return FB_OK;
}

}  // extern "C"
