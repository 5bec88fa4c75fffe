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
constexpr int kChunk = 32;           // arcs one lane walks for a row that has a lane to itself; longer rows get more lanes
constexpr int kChunkWide = 32;       // arcs one lane walks for a row spread over several lanes
constexpr size_t kLdsBytes = 160 * 1024;
constexpr size_t kLdsReserve = 1024; // reduction slots etc.
// Large graphs with float vectors whose states, clone slots and dump slot fit this many entries run a kernel
// instantiation whose LDS state buffers have this fixed length: buffer addresses are then compile-time
// constants and a gather needs no address arithmetic.
constexpr int kXsFixed = 6656;
constexpr int kXbStride = 32768;     // probability-domain kernel: bytes between its two state buffers

// One (src, weight) pair of a row of a sparse semiring matrix, as the kernels read it.
struct Arc {
    int32_t src;   // where the row gathers from: byte offset into the vector (index x element size) in a stream
                   // (StreamHost), a plain index in a sliced plan (SellHost)
    float w;       // weight (log2 units)
};

// A row with more than 64 * kChunkWide arcs is computed as several "clone" rows, each a state of its
// own in the recursion (slots after the sub-graph's K states): every clone sums a share of the
// row's arcs and takes the row's emission, every arc that leaves the row's state is repeated for
// each clone, and the state's value is the (+)-sum of its clones wherever a vector leaves the kernel.
struct CloneDesc {
    int32_t state;   // the row (local state id); it keeps the first share itself
    int32_t first;   // its further clones are slots first .. first + count - 1 (local index K + slot)
    int32_t count;
    int32_t pad_;
};

// Part of a schedule that belongs to one (sub-)graph.
struct SubDesc {
    int32_t k0;         // first state of the sub-graph in the global numbering
    int32_t K;          // its number of states
    int32_t n_slot;     // clone slots it uses
    int32_t clone0;     // its CloneDesc entries: clone0 .. clone0 + n_cdesc - 1
    int32_t n_cdesc;
    int32_t zero0;      // its rows without arcs: zero0 .. zero0 + n_zero - 1 in the zero-row list
    int32_t n_zero;
    int32_t wave_ptr0;  // host plan: where its nw + 1 slice ranges start; stream: its first WaveDesc
};

// Sliced plan of a sparse matrix-vector product in the log semifield, host side.
// A slice is 64 lanes walking arcs in lockstep.  A row with n <= kChunk arcs takes one lane; a longer
// one g lanes of one slice, g the smallest power of two with ceil(n / g) <= kChunkWide (at most 64;
// beyond that the row is cloned, see CloneDesc); all rows of a slice take the same g, the g
// partial sums of a row are combined across lanes when the slice ends.  Rows are
// sorted by length so a slice is padded little; rows without arcs are not scheduled
// at all (zero_rows).  Slices are dealt to the nw waves of a workgroup longest-first.
struct SellHost {
    int nw = 0;
    std::vector<SubDesc> sub;
    std::vector<int32_t> wave_ptr;    // slice ranges per (sub, wave)
    std::vector<int32_t> slice_trip;  // arcs each lane of the slice walks
    std::vector<int32_t> slice_lg;    // log2 of the lanes per row
    std::vector<int32_t> slice_stack; // 0: a plain slice.  2 / 4: that many slices of rows with at most 2 / exactly 1
                                      // arcs stacked into one batch of kBatchRows rows (trip = kBatchRows, lg = 0):
                                      // part t of a lane is rows [t * kBatchRows / stack, (t + 1) * kBatchRows / stack)
    std::vector<int64_t> slice_arc;   // first arc of the slice in `arcs`
    std::vector<int32_t> row_out;     // [n_slices*64*kBatchRows], entry (slice, lane, part): >= 0 target (state, or
                                      // K + clone slot) written by this lane for this part, -1 nothing (a plain
                                      // slice has part 0 only)
    std::vector<int32_t> row_vidx;    // same shape: index of the row's emission in the staged emission vector
    std::vector<Arc> arcs;            // slice-major, then step, then lane
    std::vector<CloneDesc> clones;
    std::vector<int32_t> zero_rows;   // local ids of rows without arcs
    int32_t max_slot = 0;             // most clone slots of any sub-graph
};

// rows [0, K) of a CSR-like matrix over K columns: entries ptr[r]..ptr[r+1] with column col[] and
// weight w[] (log2 units); row_vidx[r] = emission index of row r.  Appends one sub-plan to `out`.
void sell_append(SellHost &out, int32_t k0, int32_t K, const int64_t *ptr, const int32_t *col, const float *w,
                 const int32_t *row_vidx);

bool sell_in_bounds(const SellHost &S, int32_t n_vidx, std::string &why);

// ---------------------------------------------------------------------------
// Stream form of a plan: what the recursion kernel interprets.  Every wave of the
// workgroup that walks arcs owns one contiguous, cyclic stream of "rows" of 64
// entries (one per lane), grouped in batches of kBatchRows rows.  A row is 64 arcs
// (one per lane: gather, add the weight, fold into the lane's running sum), except
// that the last entry of a lane in a slice also says where the lane's finished sum
// goes: the slice's arcs are padded with zero-weight (-inf) arcs to whole batches,
// and the source field of every lane's entry in the last row of the slice's last
// batch carries the target in its upper half.  A byte of flags per batch tells
// whether it closes a slice, whether it is padding to skip, and over how many lanes
// the sums of a row are spread.  The stream of one time step is the same every
// step, so the kernel keeps it kRing-1 batches ahead of its use, across barriers
// and across steps.
//
// Stacked batches (kFlagDual, kFlagQuad; the first kMaxStacked batches of a wave's step only): the rows
// of several slices whose rows have one or two arcs share one batch, and every part carries its
// own target in the upper half of the source field of its last row (rows 1 and 3, or all four).
//
// Closing entry: src = source index (low 16 bits) | target << 16; the target is an
// index into the state buffer of the step being written, [0, K) a state, Kcap + slot
// a clone slot, Kcap + Ccap the dump slot of lanes that write nothing.  The emission
// a target takes is looked up in a table over the same index space (vix: index into
// the staged emission vector, Ecap being a slot that always holds 0).
// ---------------------------------------------------------------------------
constexpr int kBatchRows = 4;
constexpr int kRing = 3;                        // batches per unrolled iteration = prefetch ring size
constexpr int kResident = 7;                    // batches per wave and step that stay in registers (<= 8)
constexpr uint32_t kFlagInfo = 0x01;            // the batch closes a slice: its last row carries the targets
constexpr uint32_t kFlagSkip = 0x04;            // nothing to do in this batch (padding)
constexpr int kMaxStacked = 2;                  // stacked batches a wave may have: its first batches of a step
constexpr uint32_t kFlagDual = 0x40;            // with kFlagInfo: two stacked slices, rows 0-1 and rows 2-3, each closed
constexpr uint32_t kFlagQuad = 0x80;            // with kFlagInfo: four stacked slices of one row each, each closed
constexpr int kFlagLgShift = 3;                 // bits 3-5 of a closing batch: log2 of the lanes per row

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
    std::vector<Arc> arcs;
    std::vector<uint16_t> vix;         // per sub-graph, Kcap + Ccap + 1 entries: emission index of every target
    std::vector<CloneDesc> clones;
    std::vector<int32_t> zero_rows;
    int32_t Kcap = 0, Ccap = 0, Ecap = 0;   // index space of targets and emission indices (see above)
    int32_t esize = 4;                      // arc sources are index x esize
};

struct StreamDev {
    const SubDesc *sub = nullptr;
    const WaveDesc *waves = nullptr;
    const uint32_t *flagwords = nullptr;
    const Arc *arcs = nullptr;
    const uint16_t *vix = nullptr;
    const CloneDesc *clones = nullptr;
    const int32_t *zero_rows = nullptr;
};

// esize: bytes per element of the vector the kernel gathers from (4 or 8); arc sources become byte offsets
bool stream_from_sell(const SellHost &S, int32_t Kcap, int32_t Ecap, int32_t esize, StreamHost &out, std::string &why);
bool stream_in_bounds(const StreamHost &S, int32_t n_vidx, std::string &why);
// y = the (+)-product of sub-graph `sub` with x, computed on the host by walking the stream as the kernel does.
// lin: nullptr, or the arc list stream_linear_weights made of S: then the walk also checks what the multiplying
// kernel instantiation relies on (false, with the reason in why, if it does not hold).
bool stream_apply_host(const StreamHost &S, int32_t sub, const double *x, double *y, const std::vector<Arc> *lin, std::string &why);
// The arc list of S with the weights of all batches but the stacked ones replaced by 2^w, for the kernel
// instantiation that multiplies instead of adding in the exponent; arcs of weight zero-bar (padding included) get
// weight 0 and the dump slot, which always holds zero-bar, as their source, so that they never raise a running
// maximum.  False (out unspecified) if a finite weight lies outside [-kLinearSpan, kLinearSpan] (log2 units): that
// kernel normalises a row's terms by the largest gathered value alone and loses a term that lies more than 126 binary
// orders below it; with weights inside the span such a term is below 2^(2 x 50 - 126) of the row's largest product,
// i.e. below float rounding.
constexpr float kLinearSpan = 50.0f;
bool stream_linear_weights(const StreamHost &S, std::vector<Arc> &out);
constexpr float kLinWeightSpan = 64.0f, kLinRowSumTop = 40.0f;   // log2 bounds on an arc weight for the probability-domain kernel

// ---------------------------------------------------------------------------
// Plan of the probability-domain recursion kernel (fb_pstream.cpp): per arc-walking wave a sequence of units (two
// arcs per lane: three 32-bit words {source 0 | source 1 << 16, 2^w of arc 0, 2^w of arc 1}, sources = byte offsets
// into the state buffer), some of which end a slice; per slice one close word per lane {target byte offset |
// emission byte offset << 16}.
// ---------------------------------------------------------------------------
constexpr int kPChunk = 32;       // arcs one lane walks at most for a row (longer rows take more lanes)
constexpr int kPResident = 20;    // units per wave and step that stay in registers
constexpr int kPRing = 4;         // units of the streamed part in flight
// A wave's units in the order it walks them: of the first kPPatterned positions kPResident stay in registers and the
// others are re-read from L2 at every step, spread evenly behind a head of kPHead that all stay (so that the re-reading
// is spread over the step and each re-read unit can be asked for several positions ahead); what follows is all re-read.
constexpr int kPHead = 4;
constexpr int kPPatterned = 32;
constexpr bool p_streamed(int u)   // position u < kPPatterned is re-read: three of every seven behind the head
{
    return u >= kPHead && ((u - kPHead) % 7 == 1 || (u - kPHead) % 7 == 4 || (u - kPHead) % 7 == 6);
}
constexpr int p_streamed_before(int u)   // re-read positions in front of position u <= kPPatterned
{
    int n = 0;
    for (int i = 0; i < u; ++i) n += p_streamed(i) ? 1 : 0;
    return n;
}
constexpr int p_streamed_pos(int m)   // position of the m-th re-read unit, m >= 0
{
    int n = 0;
    for (int u = 0; u < kPPatterned; ++u)
        if (p_streamed(u)) {
            if (n == m) return u;
            ++n;
        }
    return kPPatterned + (m - n);
}
constexpr int p_resident_pos(int q)   // position of the q-th unit that stays in registers, q < kPResident
{
    int n = 0;
    for (int u = 0; u < kPPatterned; ++u)
        if (!p_streamed(u)) {
            if (n == q) return u;
            ++n;
        }
    return -1;
}
static_assert(kPPatterned - p_streamed_before(kPPatterned) == kPResident, "the pattern keeps kPResident units");
constexpr int kPMaxClose = 8;     // slices per wave and step
constexpr int kPMaxUnits = 128;   // units per wave and step

struct PWaveDesc {
    int64_t unit_base;            // first unit of the wave in `units` (units of 3 x 64 words)
    int32_t n_units;              // its units per time step
    int32_t n_close;              // its slices
    int32_t cw_base;              // its close words: (cw_base + c) * 64 + lane
    int32_t pad_;
    uint64_t close_mask[kPMaxUnits / 64];   // bit u: unit u ends a slice
    uint64_t lgs;                 // 3 bits per slice: log2 of the lanes its rows are spread over
};

struct PStreamHost {
    int32_t K = 0, Ccap = 0;      // states, clone slots (the dump slot is K + Ccap)
    int32_t bias = 0;             // log2 of the scale the kernel keeps its vector at (see linear_run)
    float dim = 0.0f;             // the value below which an entry that is not zero makes a run give up
    std::vector<PWaveDesc> waves; // kNWShared - 1
    std::vector<uint32_t> units;
    std::vector<uint32_t> close_words;
    std::vector<CloneDesc> clones;
    std::vector<int32_t> zero_rows;   // states without an arc of non-zero weight
};

struct PStreamDev {
    const PWaveDesc *waves = nullptr;
    const uint32_t *units = nullptr;
    const uint32_t *close_words = nullptr;
    const CloneDesc *clones = nullptr;
    const int32_t *zero_rows = nullptr;
    int32_t n_clones = 0, n_zero = 0, Ccap = 0, bias = 0;
    float dim = 0.0f;
};

// rows [0, K) of a CSR-like matrix: entries ptr[r]..ptr[r+1], column col[], weight w[] (log2 units; -inf entries are
// dropped); row_vidx[r] = emission index of row r, n_vidx = number of emission entries.  False, with the reason in
// why, if the matrix does not fit the kernel (weights out of range, too many slices, ...).
bool pstream_build(int32_t K, const int64_t *ptr, const int32_t *col, const float *w, const int32_t *row_vidx, int32_t n_vidx,
                   PStreamHost &out, std::string &why);
bool pstream_in_bounds(const PStreamHost &S, int32_t n_vidx, std::string &why);
bool pstream_apply_host(const PStreamHost &S, const double *x, double *y, int64_t *cycles, int64_t *cycles_floor, std::string &why);

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
    std::vector<uint16_t> pos;   // shared graph only: pos[k] = place of state k in `states` (its inverse)
    int32_t max_rows = 0;
};

struct PdfDev {
    const PdfSub *sub = nullptr;
    const uint16_t *row_pdf = nullptr, *row_ptr = nullptr, *states = nullptr, *pos = nullptr;
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
    fb::StreamHost h_trop;            // forward schedule of the tropical semiring, when it differs (own_trop)
    bool own_trop = false;            // the graph has parallel arcs: they combine by max there, not by (+)
    bool linear_w = false;            // the device copies of fwd / bwd carry weights as 2^w (see stream_linear_weights)
    bool linear_p = false;            // the recursions run in the probability domain (linear_run): the plans below exist
    fb::PStreamHost hp_fwd, hp_bwd;   // its plans, host
    fb::PStreamDev pfwd, pbwd;        // and device
    fb::PdfHost h_pdf;                // states grouped by pdf, for the posterior accumulation
    // device
    fb::StreamDev fwd, bwd, trop;     // trop = fwd unless own_trop
    fb::PdfDev pdfs;
    int32_t *d_pdf = nullptr;         // [K]
    float *d_init2 = nullptr;         // [K] init * log2(e)
    float *d_final2 = nullptr;        // [K] final * log2(e)
    void *leaky = nullptr;            // shared graphs: the row lists of the leaky-HMM comparison mode (fb_leaky.hip)
    std::vector<void *> allocs;       // everything to hipFree
};

namespace fb {

void set_error(const std::string &msg);
void side_stream_init();   // once per process: the streams the LF-MMI calls use beside the caller's
void static_scratch_init();   // once per device: the address of the library's built-in scratch memory
int leaky_prepare(fb_graph *g, const float *init, const float *final_);   // device tables of the leaky-HMM mode (shared graphs)
void leaky_release(fb_graph *g);
int fail(int code, const std::string &msg);

struct RecDir {
    StreamDev sched;
    const float *bound;    // start weights of this direction (init2 forward, final2 backward)
    const float *obound;   // end weights, for log Z
    void *out;             // normalised vectors, nullable: float, or the carrier type if out_carrier
    int out_carrier;       // out holds carrier-type values (workspace), not float
    double *off;           // [B][N] the shift of every stored row (accumulated offsets x out_scale), nullable
    float *cum;            // [B][N] running sums of the offsets (log2 units: stored row + cum = the true row), nullable
    double *logz;          // [B], nullable
    float out_scale;       // ln 2 for natural-log output, 1 to keep log2 units
    int32_t Ccap;          // clone slots of this direction's schedule
    int backward;
    int fill_pad;          // write -inf / 0 into the rows of padded frames
    int32_t out_ld;        // shared graph: elements between the rows of consecutive frames of out (0: the state count)
    uint16_t *bp;          // tropical semiring: back-pointers (see fb_viterbi in fb_api.cpp for the layout), else NULL
    int64_t bp_ld;         // elements per frame row of bp
    int32_t *last;         // tropical semiring: [B] local id of the best end state (-1: none)
    PStreamDev prob;       // probability-domain kernel: its plan for this direction
    int out_linear;        // ... out takes the vectors as they are kept (entry = 2^(log2 of the true value - cum)), not their logs
    int32_t *fmt;          // ... [B], nullable: 1 if the sequence's rows in out are in that form, 0 if they are logs (the run
                           //     fell back to the log form)
};

constexpr int kDoneCuts = 4;       // progress counters of a recursion launch: kDoneCuts + 1 parts by rank, the first uncounted
constexpr int kDoneStarted = 8;    // index of the `started` word in the counter block (which launch_order clears)
constexpr int kDoneNum = 6;        // ... of the word that is set when the numerator launch of an LF-MMI call has ended
constexpr int kDoneFused = 16;     // ... of the word PostParams::fused of the call's second range (written before it is read)

struct RecParams {
    RecDir dir[2];
    int n_dir;
    const int32_t *pdf;
    const float *emis;
    const int32_t *lengths;
    int32_t B, N, D, shared, Ktot;
    int32_t Kcap, Ecap;
    int32_t xs_fixed;      // kXsFixed: launch the fixed-buffer instantiation; 0: buffers sized by the graph
    int32_t linear_w;      // the streams carry weights as 2^w (fixed-buffer instantiation only)
    int32_t linear_p;      // launch the probability-domain kernel (dir[].prob)
    // A launch may cover a range of the sequences in order of length: order[r] = the sequence of rank r
    // (longest first, written by launch_order), ranks [rank0, rank0 + n_launch).  order == nullptr: all B.
    const int32_t *order;
    int32_t rank0, n_launch;
    // Progress counters (nullptr: none): a workgroup that has written everything it writes adds one to done[i],
    // i = how many of done_from[0..kDoneCuts-1] its rank (in order of length) has reached; i = 0 counts for nothing.
    // A stream can wait for such a word (hipStreamWaitValue32) and so for part of a launch.  started (nullable):
    // a word every workgroup adds one to when it begins, i.e. when it holds its compute unit.
    uint32_t *done;
    int32_t done_from[kDoneCuts];
    uint32_t *started;
};

struct PostGraph {
    PdfDev pdfs;           // states grouped by pdf
    const void *a, *b;     // normalised forward / backward vectors, float or double
    int f64;               // a, b are double
    float in_scale;        // log2(e) if a, b are natural logs, 1 if log2 units
    float sign;            // +1 / -1: how the graph's pdf posteriors enter pdf_out
    int32_t shared, Ktot;
    int32_t Kcap, Rcap;    // largest (sub-)graph: states, pdf rows
    int32_t ld;            // shared graph: elements between the rows of consecutive frames of a, b (>= K)
    float *state_post;     // nullable
    const int32_t *fmt_a, *fmt_b;   // gradient kernel, shared float graph: [B] each, nullable: 1 = the sequence's rows of a
                           // (b) hold the values themselves, 2^(log2 of the true value - cum_a (cum_b)), 0 / NULL = their logs
};

struct PostParams {
    PostGraph g[2];        // processed in order; a shared graph (one row per pdf) must come first
    int n_graph;
    const int32_t *lengths;
    int32_t B, N, D;
    float *pdf_out;        // [B][N][D], nullable
    int32_t Kcap, Kcap64, frames_per_block;   // Kcap64: largest double-carrier (sub-)graph
    const int32_t *order;  // as in RecParams: the launch covers ranks [rank0, rank0 + n_launch); nullptr: all B
    int32_t rank0, n_launch;
    // Two graphs through the gradient kernel: the running sums of the offsets of g[0]'s forward and backward rows,
    // [B][N] each, log2 units, and its log Z [B] (natural log); all three or none.
    const float *cum_a, *cum_b;
    const double *logz;
    int32_t accumulate;    // one packed graph: its pdf posteriors are added to the rows pdf_out already holds (only the
                           // entries of pdfs the sequence's graph uses are touched; padded frames are left alone)
    // A word on the device (nullable), written by launch_decide before the launch: whether the second graph's vectors
    // were complete when the launch was released.  Gradient kernel over two graphs: 0 = leave the second graph's
    // share out (a later launch in accumulate mode adds it); that later launch: not 0 = nothing is left to add.
    const int32_t *fused;
};

int launch_recursion(int nw, bool f64, bool tropical, const RecParams &p, size_t lds_bytes, void *stream);
bool recursion_fixed_available();   // the fixed-buffer instantiation (RecParams::xs_fixed) may be launched
unsigned int linear_restarts();     // diagnostic: runs the probability-domain kernel gave up and redid in the log form (synchronises)
struct BacktraceParams {
    const uint16_t *bp;      // back-pointers written by the recursion kernel
    int64_t bp_ld;           // elements per frame row
    const int32_t *last;     // [B] best end state in the kernel's index space, -1: none
    const int32_t *lengths;
    StreamDev sched;         // the forward plan (sub-graphs, clones)
    int32_t B, N, shared, Ktot, Kcap, Ccap;
    int32_t frames;          // back-pointer rows the kernel holds in LDS at a time (set by launch_backtrace)
    int32_t *path;           // [B][N]
};
int launch_backtrace(const BacktraceParams &p, void *stream);
int launch_posteriors(const PostParams &p, size_t lds_bytes, void *stream);
bool gradient_kernel_applies(const PostParams &p);
size_t gradient_lds_bytes(const PostParams &p);
int launch_gradient(const PostParams &p, size_t lds_bytes, void *stream);
bool num_add_kernel_applies(const PostParams &p);   // accumulate mode, one packed graph of small sub-graphs
int launch_num_add(const PostParams &p, void *stream);
// order[r] = index of the sequence of rank r when sorted by length (clamped to [0, N]), longest first, equal
// lengths by index
int launch_delay(void *stream);   // an empty kernel: what follows on the stream starts a launch latency later
int launch_decide(const uint32_t *count, uint32_t need, int32_t *flag, void *stream);   // *flag = *count >= need, on the device
int launch_mark(uint32_t *word, void *stream);   // *word = 1 when the stream gets there
int launch_order(const int32_t *lengths, int32_t B, int32_t N, int32_t *order, uint32_t *done, void *stream);   // done: four words to clear, or nullptr
int launch_loss(const double *logz_num, const double *logz_den, const int32_t *lengths, int32_t B, double *loss,
                void *stream);
// xs_fixed: 0, or kXsFixed for the fixed-buffer instantiation
size_t recursion_lds_bytes(int32_t Kcap, int32_t Ccap, int32_t Ecap, bool backward, bool f64, bool shared,
                           bool tropical = false, int32_t xs_fixed = 0);
size_t posterior_lds_bytes(const PostParams &p);
size_t probability_lds_bytes(int32_t D, bool staged);   // the probability-domain kernel's own use (its launch takes the larger of this and the log form's); staged: the direction keeps rows on their way out apart from the vector (backward, or rows that leave as logarithms)

}  // namespace fb
