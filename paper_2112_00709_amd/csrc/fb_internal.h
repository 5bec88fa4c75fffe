// Internal declarations shared by the host code and the kernels of libfb_amd.
#pragma once

#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "../../include/fb.h"

namespace fb {

constexpr int kWave = 64;            // gfx950 wavefront
constexpr int kNWShared = 16;        // waves per workgroup, large (sub-)graphs
constexpr int kNWSmall = 4;          // waves per workgroup, small (sub-)graphs
constexpr int kChunk = 32;           // longest arc list one lane walks; longer rows are split
constexpr size_t kLdsBytes = 160 * 1024;
constexpr size_t kLdsReserve = 1024; // reduction slots etc.

// One (src, weight) pair of a row of a sparse semiring matrix, as the kernels read it.
struct Arc {
    int32_t src;   // index into the vector the row gathers from
    float w;       // weight (log2 units in the log semiring; 1 / 0 in the plain-sum use)
};

// Part of a schedule that belongs to one (sub-)graph.
struct SubDesc {
    int32_t k0;         // first state of the sub-graph in the global numbering
    int32_t K;          // its number of states
    int32_t n_levels;   // passes over the rows: 1 + the depth of row splitting
    int32_t n_part;     // partial-result slots used by split rows
    int32_t wave_ptr0;  // where its [(n_levels * nw) + 1] slice ranges start in wave_ptr
    int32_t pad_[3];
};

// Row-split sliced-ELL schedule of a sparse matrix-vector product, host side.
// Rows are grouped 64 to a slice (one row per lane), a slice is padded to its
// longest row, rows longer than kChunk are split into partial rows that a later
// level combines, and slices are dealt to the nw waves of a workgroup so that
// every wave has about the same number of arc visits.
struct SellHost {
    int nw = 0;
    std::vector<SubDesc> sub;
    std::vector<int32_t> wave_ptr;    // slice ranges per (sub, level, wave)
    std::vector<int32_t> slice_trip;  // arcs each lane of the slice walks
    std::vector<int64_t> slice_arc;   // first arc of the slice in `arcs`
    std::vector<int32_t> row_out;     // [n_slices*64]: >=0 final row id, -1 idle lane, <=-2 partial slot -2-o
    std::vector<int32_t> row_vidx;    // [n_slices*64]: index of the row's emission in the staged emission vector
    std::vector<Arc> arcs;            // slice-major, then step, then lane
    int32_t max_part = 0;
};

// Device copy of a SellHost.
struct SellDev {
    const SubDesc *sub = nullptr;
    const int32_t *wave_ptr = nullptr;
    const int32_t *slice_trip = nullptr;
    const int64_t *slice_arc = nullptr;
    const int32_t *row_out = nullptr;
    const int32_t *row_vidx = nullptr;
    const Arc *arcs = nullptr;
};

// rows [0, n_rows) of a CSR-like matrix: entries ptr[r]..ptr[r+1] with column col[] and weight w[].
// Appends one sub-schedule to `out`.
void sell_append(SellHost &out, int32_t k0, int32_t K, int32_t n_rows, const int64_t *ptr, const int32_t *col,
                 const float *w, const int32_t *row_out_id, const int32_t *row_vidx_id, float pad_w, float one_w);

bool sell_in_bounds(const SellHost &S, int32_t n_out, int32_t n_vidx, std::string &why);
void sell_apply_host(const SellHost &S, int32_t sub, bool log_semiring, const double *x, double *y);

// ---------------------------------------------------------------------------
// Stream form of a log-semiring schedule: what the recursion kernel interprets.
// Every wave of the workgroup that walks arcs owns one contiguous, cyclic stream
// of "rows" of 64 entries (one per lane), grouped in batches of kBatchRows rows.
// A row is 64 arcs (one per lane: gather, add the weight, fold into the lane's
// running sum), except that the last row of a batch may be an info row that
// closes the slice: its entries say where each lane's finished sum goes and
// which staged emission it takes.  Slices are padded with zero-weight (-inf)
// arcs so that their info row falls on the last row of a batch.  A byte of flags
// per batch tells whether it ends with an info row, whether it is padding to
// skip, and whether a level (workgroup barrier) ends after it.  The stream of one
// time step is the same every step, so the kernel keeps it kRing-1 batches ahead
// of its use, across barriers and across steps.
//
// Info entry (in the weight field): low 16 bits = target index in the state
// buffer of the step being written, [0, K) a state, Kcap + slot a partial slot,
// Kcap + Pcap the dump slot of idle lanes; high 16 bits = index of the emission
// in the staged emission vector, Ecap being a slot that always holds 0.
// ---------------------------------------------------------------------------
constexpr int kBatchRows = 4;
constexpr int kRing = 4;                        // batches per unrolled iteration = prefetch ring size
constexpr int kResident = 6;                    // batches per wave and step that stay in registers (<= 8)
constexpr uint32_t kFlagInfo = 0x01;            // the batch's last row is an info row
constexpr uint32_t kFlagLevelEnd = 0x02;        // workgroup barrier after this batch
constexpr uint32_t kFlagSkip = 0x04;            // nothing to do in this batch (padding)

struct WaveDesc {
    int64_t arc_base;    // first entry of the wave's stream in `arcs`
    int32_t n_iter;      // unrolled iterations per time step over the streamed batches (may be 0):
                         // the wave's step is kResident + n_iter * kRing batches
    int32_t flag_base;   // its flag words (one byte per batch): two for the resident batches, then n_iter
};

struct StreamHost {
    int nw = 0;
    std::vector<SubDesc> sub;          // wave_ptr0 = index of the sub-graph's first WaveDesc
    std::vector<WaveDesc> waves;
    std::vector<uint32_t> flagwords;
    std::vector<Arc> arcs;             // info entries: src = 0, w = bits of (target16 | vidx16 << 16)
    int32_t Kcap = 0, Pcap = 0, Ecap = 0;   // index space of the info entries (see above)
};

struct StreamDev {
    const SubDesc *sub = nullptr;
    const WaveDesc *waves = nullptr;
    const uint32_t *flagwords = nullptr;
    const Arc *arcs = nullptr;
};

bool stream_from_sell(const SellHost &S, int32_t Kcap, int32_t Ecap, StreamHost &out, std::string &why);
bool stream_in_bounds(const StreamHost &S, int32_t n_vidx, std::string &why);
void stream_apply_host(const StreamHost &S, int32_t sub, const double *x, double *y);

// States grouped by pdf for the posterior accumulation: per (sub-)graph, one row per pdf it uses
// (every pdf for a shared graph), listing the local ids of the states tied to it.  16-bit entries:
// a workgroup keeps its graph's table in LDS.
struct PdfSub {
    int32_t k0, K;        // the sub-graph's first state and state count
    int32_t row0, n_rows; // its rows in row_pdf
    int32_t ptr0;         // its n_rows + 1 offsets in row_ptr (relative to st0)
    int32_t st0;          // its K entries in states
    int32_t pad_[2];
};

struct PdfHost {
    std::vector<PdfSub> sub;
    std::vector<uint16_t> row_pdf, row_ptr, states;
    int32_t max_rows = 0;
};

struct PdfDev {
    const PdfSub *sub = nullptr;
    const uint16_t *row_pdf = nullptr, *row_ptr = nullptr, *states = nullptr;
};

struct HostLayout {                   // the graph-layout step, kept for fb_graph_layout
    std::vector<int32_t> in_ptr, in_src, in_perm, out_ptr, out_dst, out_perm, pdf_ptr, pdf_states;
    std::vector<float> in_w, out_w;
};

}  // namespace fb

struct fb_graph {
    int32_t K = 0, D = 0, n_seq = 0;  // n_seq == 0: shared
    int64_t E = 0;
    int nw = 0;                       // waves per workgroup its schedules were built for
    int32_t max_sub_K = 0;
    bool host_only = false;
    bool f64 = false;                 // state vectors carried in double (exponentials stay single)
    fb::HostLayout lay;
    std::vector<int32_t> state_off;   // packed only
    fb::StreamHost h_fwd, h_bwd;      // host schedules of the two recursions
    fb::PdfHost h_pdf;                // states grouped by pdf, for the posterior accumulation
    // device
    fb::StreamDev fwd, bwd;
    fb::PdfDev pdfs;
    int32_t *d_pdf = nullptr;         // [K]
    float *d_init2 = nullptr;         // [K] init * log2(e)
    float *d_final2 = nullptr;        // [K] final * log2(e)
    std::vector<void *> allocs;       // everything to hipFree
};

namespace fb {

void set_error(const std::string &msg);
void side_stream_init();   // once per process: the stream lfmmi_loss_grad runs the numerator launch on
int fail(int code, const std::string &msg);

struct RecDir {
    StreamDev sched;
    const float *bound;    // start weights of this direction (init2 forward, final2 backward)
    const float *obound;   // end weights, for log Z
    void *out;             // normalised vectors, nullable: float, or the carrier type if out_carrier
    int out_carrier;       // out holds carrier-type values (workspace), not float
    float *off;            // [B][N] offsets, nullable
    double *logz;          // [B], nullable
    float out_scale;       // ln 2 for natural-log output, 1 to keep log2 units
    int32_t Pcap;          // partial slots of this direction's schedule
    int backward;
    int fill_pad;          // write -inf / 0 into the rows of padded frames
};

struct RecParams {
    RecDir dir[2];
    int n_dir;
    const int32_t *pdf;
    const float *emis;
    const int32_t *lengths;
    int32_t B, N, D, shared, Ktot;
    int32_t Kcap, Ecap;
};

struct PostGraph {
    PdfDev pdfs;           // states grouped by pdf
    const void *a, *b;     // normalised forward / backward vectors, float or double
    int f64;               // a, b are double
    float in_scale;        // log2(e) if a, b are natural logs, 1 if log2 units
    float sign;            // +1 / -1: how the graph's pdf posteriors enter pdf_out
    int32_t shared, Ktot;
    int32_t Kcap, Rcap;    // largest (sub-)graph: states, pdf rows
    float *state_post;     // nullable
};

struct PostParams {
    PostGraph g[2];        // processed in order; a shared graph (one row per pdf) must come first
    int n_graph;
    const int32_t *lengths;
    int32_t B, N, D;
    float *pdf_out;        // [B][N][D], nullable
    int32_t Kcap, Kcap64, frames_per_block;   // Kcap64: largest double-carrier (sub-)graph
};

int launch_recursion(int nw, bool f64, const RecParams &p, size_t lds_bytes, void *stream);
int launch_posteriors(const PostParams &p, size_t lds_bytes, void *stream);
int launch_loss(const double *logz_num, const double *logz_den, const int32_t *lengths, int32_t B, double *loss,
                void *stream);
size_t recursion_lds_bytes(int32_t Kcap, int32_t Pcap, int32_t Ecap, bool backward, bool f64, bool shared);
size_t posterior_lds_bytes(const PostParams &p);

}  // namespace fb
