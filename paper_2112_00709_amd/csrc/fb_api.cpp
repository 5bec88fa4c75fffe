// The compute entry points of the C ABI: argument checks and kernel launches.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstdlib>
#include <mutex>
#include <string>

#include "fb_internal.h"

using namespace fb;

namespace {

constexpr float kLn2f = 0.69314718055994530942f;
constexpr float kLog2ef = 1.44269504088896340736f;

int check_common(const char *who, const fb_graph *g, const void *p1, const void *p2, int32_t B, int32_t N, int32_t D)
{
    const std::string w(who);
    if (!g) return fail(FB_EINVAL, w + ": graph is NULL");
    if (g->host_only) return fail(FB_EINVAL, w + ": graph was created with FB_GRAPH_HOST_ONLY");
    if (!p1 || !p2) return fail(FB_EINVAL, w + ": NULL input array");
    if (B <= 0 || N <= 0 || D <= 0) return fail(FB_EINVAL, w + ": B, N and D must be positive");
    if (D != g->D) return fail(FB_EINVAL, w + ": D differs from the graph's D");
    if (g->n_seq > 0 && B != g->n_seq) return fail(FB_EINVAL, w + ": B differs from the number of packed graphs");
    return FB_OK;
}

RecDir make_dir(const fb_graph *g, bool backward, void *out, bool out_carrier, double *off, double *logz,
                float out_scale, bool fill_pad)
{
    RecDir r{};
    r.sched = backward ? g->bwd : g->fwd;
    r.bound = backward ? g->d_final2 : g->d_init2;
    r.obound = backward ? g->d_init2 : g->d_final2;
    r.out = out;
    r.out_carrier = out_carrier ? 1 : 0;
    r.off = off;
    r.logz = logz;
    r.out_scale = out_scale;
    r.Ccap = backward ? g->h_bwd.Ccap : g->h_fwd.Ccap;
    r.backward = backward ? 1 : 0;
    r.fill_pad = fill_pad ? 1 : 0;
    r.prob = backward ? g->pbwd : g->pfwd;
    return r;
}

// A range of the sequences in order of length (RecParams::order); order == nullptr: all of them.
struct RankRange {
    const int32_t *order = nullptr;
    int32_t rank0 = 0, count = 0;
};

int run_recursion(const fb_graph *g, const float *emis, const int32_t *lengths, int32_t B, int32_t N, int32_t D,
                  const RecDir *dirs, int n_dir, fb_stream stream, bool tropical = false, RankRange range = RankRange(),
                  uint32_t *done = nullptr, const int32_t *done_from = nullptr, bool count_started = false)
{
    RecParams p{};
    p.done = done_from ? done : nullptr;
    for (int i = 0; i < kDoneCuts; ++i) p.done_from[i] = done_from ? done_from[i] : 0;
    p.started = (done && count_started) ? done + kDoneStarted : nullptr;
    p.order = range.order;
    p.rank0 = range.rank0;
    p.n_launch = range.count;
    p.n_dir = n_dir;
    p.pdf = g->d_pdf;
    p.emis = emis;
    p.lengths = lengths;
    p.B = B; p.N = N; p.D = D;
    p.shared = g->n_seq == 0;
    p.Ktot = g->K;
    p.Kcap = g->max_sub_K;
    p.Ecap = p.shared ? D : g->max_sub_K;
    size_t lds = 0;
    for (int i = 0; i < n_dir; ++i) {
        p.dir[i] = dirs[i];
        lds = std::max(lds, recursion_lds_bytes(p.Kcap, dirs[i].Ccap, p.Ecap, dirs[i].backward != 0, g->f64, p.shared != 0,
                                                tropical));
    }
    if (lds > kLdsBytes) return fail(FB_EUNSUPPORTED, "state vectors and emission rows exceed the on-chip memory");
    // large graphs with float vectors: the instantiation with fixed-length state buffers, when everything fits them
    // (the tropical instantiation keeps sized buffers: with fixed ones it runs out of registers)
    if (g->nw == kNWShared && !g->f64 && !tropical && recursion_fixed_available()) {
        size_t lds_fixed = 0;
        bool fits = true;
        for (int i = 0; i < n_dir; ++i) {
            fits = fits && p.Kcap + dirs[i].Ccap + 1 <= kXsFixed;
            lds_fixed = std::max(lds_fixed, recursion_lds_bytes(p.Kcap, dirs[i].Ccap, p.Ecap, dirs[i].backward != 0, false,
                                                                p.shared != 0, tropical, kXsFixed));
        }
        if (fits && lds_fixed <= kLdsBytes) {
            p.xs_fixed = kXsFixed;
            lds = lds_fixed;
        }
    }
    // graphs that run in the probability domain were found to fit the fixed buffers when they were created
    if (g->linear_p && !tropical) {
        if (!p.xs_fixed) return fail(FB_EHIP, "internal error: probability-domain kernel without fixed buffers");
        p.linear_p = 1;
    }
    // graphs whose streams carry weights as 2^w were found to fit the fixed buffers when they were created
    if (g->linear_w && !tropical) {
        if (!p.xs_fixed) return fail(FB_EHIP, "internal error: linear weights without fixed buffers");
        p.linear_w = 1;
    }
    return launch_recursion(g->nw, g->f64, tropical, p, lds, stream);
}

PostGraph make_post(const fb_graph *g, const void *a, const void *b, bool f64, float in_scale, float sign, float *state_post)
{
    PostGraph q{};
    q.pdfs = g->pdfs;
    q.a = a;
    q.b = b;
    q.f64 = f64 ? 1 : 0;
    q.in_scale = in_scale;
    q.sign = sign;
    q.shared = g->n_seq == 0;
    q.Ktot = g->K;
    q.Kcap = g->max_sub_K;
    q.Rcap = g->h_pdf.max_rows;
    q.ld = g->K;
    q.state_post = state_post;
    return q;
}

// what the gradient kernel needs beside the vectors (PostParams::cum_a, cum_b, logz); all null: not given
struct Offsets {
    const float *cum_a = nullptr, *cum_b = nullptr;
    const double *logz = nullptr;
    const int32_t *fused = nullptr;   // PostParams::fused
};

int run_posteriors(const PostGraph *gs, int n_graph, const int32_t *lengths, int32_t B, int32_t N, int32_t D,
                   float *pdf_out, fb_stream stream, RankRange range = RankRange(), bool accumulate = false,
                   Offsets offs = Offsets())
{
    PostParams p{};
    p.accumulate = accumulate ? 1 : 0;
    if (offs.cum_a && offs.cum_b && offs.logz) { p.cum_a = offs.cum_a; p.cum_b = offs.cum_b; p.logz = offs.logz; }
    p.fused = offs.fused;
    p.order = range.order;
    p.rank0 = range.rank0;
    p.n_launch = range.count;
    p.n_graph = n_graph;
    for (int i = 0; i < n_graph; ++i) {
        p.g[i] = gs[i];
        p.Kcap = std::max(p.Kcap, gs[i].Kcap);
        if (gs[i].f64) p.Kcap64 = std::max(p.Kcap64, (gs[i].Kcap + 1) & ~1);   // even: what follows stays 16-byte aligned
    }
    p.lengths = lengths;
    p.B = B; p.N = N; p.D = D;
    p.pdf_out = pdf_out;
    p.frames_per_block = 6;
    if (gradient_kernel_applies(p)) {   // shared float denominator + small packed numerators: the specialised kernel
        const size_t glds = gradient_lds_bytes(p);
        if (glds <= kLdsBytes) return launch_gradient(p, glds, stream);
    }
    if (num_add_kernel_applies(p)) {
        // (a launch that may find nothing left to add, PostParams::fused, comes in few workgroups: they are all dispatched
        // beside the call's last gradient launch before they can leave)
        p.frames_per_block = p.fused ? 32 : 8;
        return launch_num_add(p, stream);
    }
    const size_t lds = posterior_lds_bytes(p);
    if (lds > kLdsBytes) return fail(FB_EUNSUPPORTED, "state vector, pdf row and pdf tables exceed the on-chip memory");
    return launch_posteriors(p, lds, stream);
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Whether every launch that reads the denominator's vectors in an LF-MMI call of this shape is one of the gradient
// kernel (run_posteriors decides the same way): both graphs together, or the denominator alone.
bool gradient_reads_denominator(const PostGraph *q, const int32_t *lengths, int32_t B, int32_t N, int32_t D, float *grad)
{
    const float dummy_f = 0.0f;
    const double dummy_d = 0.0;
    for (int n_graph = 1; n_graph <= 2; ++n_graph) {
        PostParams p{};
        p.cum_a = p.cum_b = &dummy_f;   // (only tested for presence)
        p.logz = &dummy_d;
        p.n_graph = n_graph;
        for (int i = 0; i < n_graph; ++i) {
            p.g[i] = q[i];
            p.Kcap = std::max(p.Kcap, q[i].Kcap);
        }
        p.lengths = lengths;
        p.B = B; p.N = N; p.D = D;
        p.pdf_out = grad;
        p.frames_per_block = 6;
        if (!gradient_kernel_applies(p) || gradient_lds_bytes(p) > kLdsBytes) return false;
    }
    return true;
}

// First rank of length group i + 1 of B sequences in order of length (see lfmmi_loss_grad).
int32_t group_cut(int32_t B, int i, bool fills_chip)
{
    static const double frac[3] = {0.25, 0.50, 0.97};
    // Workgroups of a launch go round the 8 XCDs of the chip by index, starting at the first, and inside an XCD
    // round its 4 shader engines; a workgroup waits for a compute unit of the engine it is sent to even while
    // others are free elsewhere.  The first two ranges therefore take multiples of 16 sequences (32 workgroups)
    // when the batch fills the chip (two workgroups per sequence), the last cut a multiple of 4 sequences (8 workgroups):
    // every engine then gets the same number of workgroups over all launches.  (Measured on a batch of 128:
    // ranges of 24 / 40 / 60 / 4 sequences instead of 32 / 32 / 60 / 4 leave a workgroup of the third range
    // waiting until one of the shortest sequences has finished, and that range ends 0.6 - 0.9 ms late.)
    const int32_t g = (i < 2 && fills_chip) ? 16 : 4;
    const int32_t c = ((int32_t)(frac[i] * B + 0.5) + g / 2) / g * g;
    return std::min(std::max(c, g * (i + 1)), (B - 4 * (3 - i)) / 4 * 4);
}

// stage timing of lfmmi_loss_grad (fb_profile_enable / fb_profile_read)
struct Profile {
    bool on = false, recorded = false;
    hipEvent_t ev[7] = {};   // 0-4 on the caller's stream, 5-6 around the numerator launch on the side stream
} g_prof;

void mark(int i, hipStream_t stream)
{
    if (g_prof.on) (void)hipEventRecord(g_prof.ev[i], stream);
}

// Three further streams (default priority) and untimed events, created once per process by
// side_stream_init, which fb_graph_create calls when it makes a packed graph (the numerators of an LF-MMI call: only
// those calls use the streams, and a process that runs recursions of a shared graph on streams of its own keeps the
// hardware queues for them), so that compute calls themselves never allocate.
// With the caller's stream that makes four, the number of hardware queues a process has: one per length
// group of lfmmi_loss_grad (group 0, the longest sequences, on the caller's stream).  `stream` (= group[0])
// also takes the numerator launch of a call too small for groups.  Setting FB_AMD_SERIAL=1 in the
// environment keeps everything on the caller's stream.
constexpr int kGroups = 4;
constexpr int kRange0Parts = 2;   // the longest range is cut once more (see lfmmi_run)
struct SideStream {
    bool ok = false, tried = false;
    bool groups_ok = false;                     // the group streams exist (FB_AMD_GROUPS=0 in the environment: they do not)
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    int n_cu = 0;                               // compute units of the device
    bool can_wait_value = false;                // hipStreamWaitValue32 is available on the device
    hipStream_t group[kGroups - 1] = {};
    hipEvent_t num_done = nullptr;              // the numerator launch has finished
    hipEvent_t group_done[kGroups - 1] = {};    // a side group's gradient launch has finished
};

SideStream &side_stream()
{
    static SideStream s;
    return s;
}


// Scratch memory of lfmmi_loss_grad_static: part of the library's image on every GPU it runs on, so a call needs no
// allocation.  In host code the array's name only stands for the symbol; the address on a GPU is looked up once per
// device, with that device current, and kept.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
struct StaticScratch {
    std::mutex lock;
    void *ptr[kMaxDevices] = {};
} g_scratch;

// The address of the scratch array on the current device (nullptr and an error message on failure).
void *static_scratch()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        fail(FB_EHIP, "lfmmi_loss_grad_static: no current device");
        return nullptr;
    }
    std::lock_guard<std::mutex> hold(g_scratch.lock);
    if (!g_scratch.ptr[dev]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) {
            fail(FB_EHIP, std::string("lfmmi_loss_grad_static: hipGetSymbolAddress: ") + hipGetErrorString(e));
            return nullptr;
        }
        g_scratch.ptr[dev] = p;
    }
    return g_scratch.ptr[dev];
}

}  // namespace

namespace fb {

void static_scratch_init() { (void)static_scratch(); }   // set-up time, this device current: later calls find the address

void side_stream_init()
{
    SideStream &s = side_stream();
    if (s.tried) return;
    s.tried = true;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&s.n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        s.n_cu = 0;
    int can = 0;
    s.can_wait_value = hipDeviceGetAttribute(&can, hipDeviceAttributeCanUseStreamWaitValue, dev) == hipSuccess && can == 1;
    const char *serial = getenv("FB_AMD_SERIAL");
    if (serial && serial[0] == '1') return;
    if (hipEventCreateWithFlags(&s.fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&s.join, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&s.num_done, hipEventDisableTiming) != hipSuccess)
        return;
    if (hipStreamCreateWithFlags(&s.group[0], hipStreamNonBlocking) != hipSuccess) return;
    s.stream = s.group[0];
    s.ok = true;
    // A process has four hardware queues: a caller who runs work of its own on further streams beside this
    // library's may prefer to keep them (then lfmmi_loss_grad_ragged works like lfmmi_loss_grad).
    const char *groups = getenv("FB_AMD_GROUPS");
    if (groups && groups[0] == '0') return;
    if (hipEventCreateWithFlags(&s.group_done[0], hipEventDisableTiming) != hipSuccess) return;
    for (int i = 1; i < kGroups - 1; ++i)
        if (hipStreamCreateWithFlags(&s.group[i], hipStreamNonBlocking) != hipSuccess ||
            hipEventCreateWithFlags(&s.group_done[i], hipEventDisableTiming) != hipSuccess)
            return;
    s.groups_ok = true;
}

}  // namespace fb

extern "C" {

int fb_profile_enable(int on)
{
    if (on && !g_prof.on) {
        for (int i = 0; i < 7; ++i)
            if (hipEventCreate(&g_prof.ev[i]) != hipSuccess) {
                for (int j = 0; j < i; ++j) (void)hipEventDestroy(g_prof.ev[j]);
                return fail(FB_EHIP, "fb_profile_enable: hipEventCreate failed");
            }
        g_prof.on = true;
        g_prof.recorded = false;
    } else if (!on && g_prof.on) {
        for (int i = 0; i < 7; ++i) (void)hipEventDestroy(g_prof.ev[i]);
        g_prof.on = false;
        g_prof.recorded = false;
    }
    return FB_OK;
}

int fb_profile_read(float *ms)
{
    if (!g_prof.on || !g_prof.recorded || !ms) return fail(FB_EINVAL, "fb_profile_read: nothing recorded");
    if (hipEventSynchronize(g_prof.ev[4]) != hipSuccess) return fail(FB_EHIP, "fb_profile_read: hipEventSynchronize failed");
    if (hipEventSynchronize(g_prof.ev[6]) != hipSuccess) return fail(FB_EHIP, "fb_profile_read: hipEventSynchronize failed");
    const int first[4] = {5, 1, 2, 3}, last[4] = {6, 2, 3, 4};
    for (int i = 0; i < 4; ++i)
        if (hipEventElapsedTime(&ms[i], g_prof.ev[first[i]], g_prof.ev[last[i]]) != hipSuccess)
            return fail(FB_EHIP, "fb_profile_read: hipEventElapsedTime failed");
    return FB_OK;
}

}  // extern "C"

extern "C" {

int fb_alpha(const fb_graph *g, const float *emis, const int32_t *lengths, int32_t B, int32_t N, int32_t D, float *alpha,
             double *alpha_cum, double *logz, fb_stream stream)
{
    int rc = check_common("fb_alpha", g, emis, lengths, B, N, D);
    if (rc) return rc;
    const RecDir d = make_dir(g, false, alpha, false, alpha_cum, logz, kLn2f, true);
    return run_recursion(g, emis, lengths, B, N, D, &d, 1, stream);
}

int fb_beta(const fb_graph *g, const float *emis, const int32_t *lengths, int32_t B, int32_t N, int32_t D, float *beta,
            double *beta_cum, double *logz, fb_stream stream)
{
    int rc = check_common("fb_beta", g, emis, lengths, B, N, D);
    if (rc) return rc;
    const RecDir d = make_dir(g, true, beta, false, beta_cum, logz, kLn2f, true);
    return run_recursion(g, emis, lengths, B, N, D, &d, 1, stream);
}

int fb_posteriors(const fb_graph *g, const float *alpha, const float *beta, const int32_t *lengths, int32_t B, int32_t N,
                  int32_t D, float *state_post, float *pdf_post, fb_stream stream)
{
    int rc = check_common("fb_posteriors", g, alpha, beta, B, N, D);
    if (rc) return rc;
    if (!lengths) return fail(FB_EINVAL, "fb_posteriors: lengths is NULL");
    if (!state_post && !pdf_post) return fail(FB_EINVAL, "fb_posteriors: no output requested");
    const PostGraph q = make_post(g, alpha, beta, false, kLog2ef, 1.0f, state_post);
    return run_posteriors(&q, 1, lengths, B, N, D, pdf_post, stream);
}

// Back-pointer rows: per frame the states and, behind them, the clone slots of the forward plan.
// shared graph: [B][N][K + Ccap]; packed graphs: [N][K + n_seq * Ccap] (sequence b: its state columns, then
// its Ccap clone columns at K + b * Ccap).
static size_t viterbi_bp_ld(const fb_graph *g)
{
    // (a multiple of 8 entries: rows start on 16-byte boundaries, which the back-trace copies in 16-byte pieces)
    return ((size_t)g->K + (size_t)(g->n_seq == 0 ? 1 : g->n_seq) * (size_t)(g->own_trop ? g->h_trop : g->h_fwd).Ccap + 7) & ~(size_t)7;
}

size_t fb_viterbi_workspace_bytes(const fb_graph *g, int32_t B, int32_t N)
{
    if (!g || B <= 0 || N <= 0) return 0;
    const size_t rows = (g->n_seq == 0 ? (size_t)B * N : (size_t)N) * viterbi_bp_ld(g);
    return align256(rows * sizeof(uint16_t)) + align256((size_t)B * sizeof(int32_t));
}

int fb_viterbi(const fb_graph *g, const float *emis, const int32_t *lengths, int32_t B, int32_t N, int32_t D, double *score,
               int32_t *path, void *ws, size_t ws_bytes, fb_stream stream)
{
    int rc = check_common("fb_viterbi", g, emis, lengths, B, N, D);
    if (rc) return rc;
    if (!score || !path) return fail(FB_EINVAL, "fb_viterbi: score or path is NULL");
    if (!ws || ws_bytes < fb_viterbi_workspace_bytes(g, B, N)) return fail(FB_EINVAL, "fb_viterbi: workspace missing or too small");
    if (((uintptr_t)ws & 255) != 0) return fail(FB_EINVAL, "fb_viterbi: workspace must be 256-byte aligned");
    const size_t rows = (g->n_seq == 0 ? (size_t)B * N : (size_t)N) * viterbi_bp_ld(g);
    uint16_t *bp = (uint16_t *)ws;
    int32_t *last = (int32_t *)((char *)ws + align256(rows * sizeof(uint16_t)));
    RecDir d = make_dir(g, false, nullptr, false, nullptr, score, 1.0f, false);
    d.sched = g->trop;
    d.Ccap = (g->own_trop ? g->h_trop : g->h_fwd).Ccap;
    d.bp = bp;
    d.bp_ld = (int64_t)viterbi_bp_ld(g);
    d.last = last;
    if ((rc = run_recursion(g, emis, lengths, B, N, D, &d, 1, stream, true))) return rc;
    BacktraceParams bt{};
    bt.bp = bp; bt.bp_ld = d.bp_ld; bt.last = last; bt.lengths = lengths; bt.sched = g->trop;
    bt.B = B; bt.N = N; bt.shared = g->n_seq == 0; bt.Ktot = g->K; bt.Kcap = g->max_sub_K; bt.Ccap = d.Ccap;
    bt.path = path;
    return launch_backtrace(bt, stream);
}

// rows of the denominator's workspace vectors start on 16-byte boundaries
static size_t lfmmi_den_ld(const fb_graph *den) { return ((size_t)den->K + 3) & ~(size_t)3; }

size_t fb_lfmmi_workspace_bytes(const fb_graph *den, const fb_graph *num, int32_t B, int32_t N, int32_t D)
{
    if (!den || !num || B <= 0 || N <= 0 || D <= 0) return 0;
    const size_t den_vec = align256((size_t)B * N * lfmmi_den_ld(den) * (den->f64 ? 8 : 4));
    const size_t num_vec = align256((size_t)N * num->K * (num->f64 ? 8 : 4));
    const size_t z = align256((size_t)B * sizeof(double));
    const size_t cum = align256((size_t)B * N * sizeof(float));   // running offsets of the denominator rows, per direction
    // + the sequences in order of length, a progress counter, the form of every sequence's forward and backward rows
    return 2 * den_vec + 2 * num_vec + 2 * z + align256((size_t)B * sizeof(int32_t)) + 2 * cum + 256 + 2 * align256((size_t)B * sizeof(int32_t));
}

// in_groups: run the batch as ranges of sequences by length; num_apart: the numerators' share of the gradient in a
// launch of its own (see below)
static int lfmmi_run(const fb_graph *den, const fb_graph *num, const float *emis, const int32_t *lengths, int32_t B,
                     int32_t N, int32_t D, double *loss, double *logz_num, double *logz_den, float *grad, void *ws,
                     size_t ws_bytes, fb_stream stream, bool in_groups, bool num_apart)
{
    int rc = check_common("lfmmi_loss_grad", den, emis, lengths, B, N, D);
    if (rc) return rc;
    if ((rc = check_common("lfmmi_loss_grad", num, emis, lengths, B, N, D))) return rc;
    if (den->n_seq != 0) return fail(FB_EINVAL, "lfmmi_loss_grad: the denominator graph must be shared");
    if (num->n_seq == 0) return fail(FB_EINVAL, "lfmmi_loss_grad: the numerator graphs must be packed");
    if (!loss || !grad) return fail(FB_EINVAL, "lfmmi_loss_grad: loss or grad is NULL");
    const size_t need = fb_lfmmi_workspace_bytes(den, num, B, N, D);
    if (!ws || ws_bytes < need) return fail(FB_EINVAL, "lfmmi_loss_grad: workspace missing or too small");
    if (((uintptr_t)ws & 255) != 0) return fail(FB_EINVAL, "lfmmi_loss_grad: workspace must be 256-byte aligned");
    // The library's streams, their events and the stage timer are the process's: one call at a time enqueues its
    // work (events are recorded and waited for in pairs inside a call, so calls must not interleave there).
    static std::mutex enqueue_lock;
    std::lock_guard<std::mutex> hold(enqueue_lock);

    // workspace: forward and backward vectors of both graphs in log2 units, log Z when the caller keeps none, the
    // sequences in order of length, the running offsets of the denominator's forward and backward rows
    char *w = (char *)ws;
    const size_t den_vec = align256((size_t)B * N * lfmmi_den_ld(den) * (den->f64 ? 8 : 4));
    const size_t num_vec = align256((size_t)N * num->K * (num->f64 ? 8 : 4));
    void *den_a = w; w += den_vec;
    void *den_b = w; w += den_vec;
    void *num_a = w; w += num_vec;
    void *num_b = w; w += num_vec;
    double *zn = logz_num ? logz_num : (double *)w; w += align256((size_t)B * sizeof(double));
    double *zd = logz_den ? logz_den : (double *)w; w += align256((size_t)B * sizeof(double));
    int32_t *order = (int32_t *)w; w += align256((size_t)B * sizeof(int32_t));
    float *cum_a = (float *)w; w += align256((size_t)B * N * sizeof(float));
    float *cum_b = (float *)w; w += align256((size_t)B * N * sizeof(float));
    uint32_t *done = (uint32_t *)w; w += 256;
    int32_t *fmt_a = (int32_t *)w; w += align256((size_t)B * sizeof(int32_t));
    int32_t *fmt_b = (int32_t *)w;

    // Both recursions of a graph run side by side in one launch.  The denominator launch goes first on
    // the caller's stream; the (much smaller) numerator launch runs beside it on the library's side stream
    // and fills compute units as short sequences of the denominator finish.
    RecDir dn[2] = {make_dir(num, false, num_a, true, nullptr, zn, 1.0f, false),
                    make_dir(num, true, num_b, true, nullptr, nullptr, 1.0f, false)};
    RecDir dd[2] = {make_dir(den, false, den_a, true, nullptr, zd, 1.0f, false),
                    make_dir(den, true, den_b, true, nullptr, nullptr, 1.0f, false)};
    dd[0].out_ld = dd[1].out_ld = (int32_t)lfmmi_den_ld(den);
    dd[0].cum = cum_a;
    dd[1].cum = cum_b;
    Offsets offs;
    offs.cum_a = cum_a; offs.cum_b = cum_b; offs.logz = zd;
    hipStream_t main_s = (hipStream_t)stream;
    SideStream &side = side_stream();
    // Eq. 17: numerator pdf posteriors minus denominator pdf posteriors
    PostGraph q[2] = {make_post(den, den_a, den_b, den->f64, 1.0f, -1.0f, nullptr),
                      make_post(num, num_a, num_b, num->f64, 1.0f, 1.0f, nullptr)};
    q[0].ld = (int32_t)lfmmi_den_ld(den);
    // A denominator that runs in the probability domain leaves its vectors as they are kept (no logarithms on the
    // way out) when it is the gradient kernel that reads them; which sequences' rows have that form (all but those
    // that fell back to the log form) it says per sequence and direction.
    if (den->linear_p && gradient_reads_denominator(q, lengths, B, N, D, grad)) {
        dd[0].out_linear = dd[1].out_linear = 1;
        dd[0].fmt = fmt_a;
        dd[1].fmt = fmt_b;
        q[0].fmt_a = fmt_a;
        q[0].fmt_b = fmt_b;
    }

    hipStreamCaptureStatus cap_state = hipStreamCaptureStatusNone;
    const bool not_capturing = hipStreamIsCapturing(main_s, &cap_state) == hipSuccess && cap_state == hipStreamCaptureStatusNone;
    if (in_groups && side.groups_ok && B >= 8 * kGroups && side.can_wait_value && not_capturing) {
        // Length groups by progress counters.  A sequence's gradient needs only that sequence's vectors, and the
        // sequences of a batch differ in length, so the compute units of the short ones would idle until the
        // longest denominator recursion ends.  The denominator recursions of the whole batch are one launch with
        // its workgroups in order of length, longest first; the batch is cut into kGroups ranges of ranks (the
        // first once more in two), each with a progress counter that the recursion workgroups of the range
        // increment when they are done, and every range has a gradient launch of its own that waits for its
        // counter (a stream wait on the word) and then runs on the compute units its sequences have left.  Only
        // the gradient of the very longest sequences waits for the launch itself and is all that is left when it
        // ends.  Nothing here depends on the lengths themselves, only on ranks, which the device computes.
        // A denominator workgroup fills a compute unit, so none of this work shares a compute unit with the
        // longest sequences, which set the time of the call.  The numerators of all sequences are one launch that
        // waits until the denominator workgroups hold their compute units (a word they add to when they begin):
        // launched at once it would take compute units before every denominator workgroup has one.
        const bool fills = side.n_cu > 0 && 2 * (int64_t)B >= side.n_cu;
        const int32_t cut[kGroups + 1] = {0, group_cut(B, 0, fills), group_cut(B, 1, fills), group_cut(B, 2, fills), B};
        hipStream_t gs[kGroups] = {main_s, side.group[0], side.group[1], side.group[2]};
        auto ok = [](hipError_t e) { return e == hipSuccess; };
        mark(0, main_s);
        if ((rc = launch_order(lengths, B, N, order, done, main_s))) return rc;
        if (!ok(hipEventRecord(side.fork, main_s))) return fail(FB_EHIP, "lfmmi_loss_grad: event record failed");
        for (int g = 1; g < kGroups; ++g)
            if (!ok(hipStreamWaitEvent(gs[g], side.fork, 0))) return fail(FB_EHIP, "lfmmi_loss_grad: stream wait failed");
        mark(1, main_s);
        // From here on the side streams hold work of this call: whatever happens, the caller's stream waits
        // for them before the call returns.
        const int32_t part1 = cut[1] >= 4 * kRange0Parts ? cut[1] / 2 : cut[1];   // the longest range, cut once more
        const int32_t from[kDoneCuts] = {part1, cut[1], cut[2], cut[3]};
        const int32_t upto[kDoneCuts] = {cut[1], cut[2], cut[3], B};
        auto slot_range = [&](int slot) { return RankRange{order, from[slot - 1], upto[slot - 1] - from[slot - 1]}; };
        auto wait_slot = [&](hipStream_t st, int slot) {   // every recursion workgroup (two per sequence) of the slot's ranks is done
            const uint32_t n = 2u * (uint32_t)(upto[slot - 1] - from[slot - 1]);
            return n == 0 || ok(hipStreamWaitValue32(st, done + slot, n, hipStreamWaitValueGte, 0xffffffffu));
        };
        bool decides_on_device = gradient_reads_denominator(q, lengths, B, N, D, grad);
        {
            PostParams pa{};
            pa.n_graph = 1;
            pa.g[0] = q[1];
            pa.accumulate = 1;
            pa.pdf_out = grad;
            decides_on_device = decides_on_device && num_add_kernel_applies(pa);
        }
        auto stages = [&]() -> int {
            int r;
            if ((r = run_recursion(den, emis, lengths, B, N, D, dd, 2, main_s, false, RankRange{order, 0, B}, done, from, true))) return r;
            mark(2, main_s);
            hipStream_t ns = gs[kGroups - 1];
            const uint32_t holding = side.n_cu > 0 ? (uint32_t)std::min<int64_t>(2 * (int64_t)B, side.n_cu) : 1u;
            if (!ok(hipStreamWaitValue32(ns, done + kDoneStarted, holding, hipStreamWaitValueGte, 0xffffffffu)))
                return fail(FB_EHIP, "lfmmi_loss_grad: stream wait on a value failed");
            mark(5, ns);
            if ((r = run_recursion(num, emis, lengths, B, N, D, dn, 2, ns, false, RankRange{order, 0, B}))) return r;
            // (a word on the device says that the launch has ended: see the second range below.  A launch of its own
            // behind it, not a count by the numerator workgroups: each of those would have to push its rows out of
            // its L2 before it counts, 256 times beside the denominator launch.)
            uint32_t *num_ended = done + kDoneNum;
            if (decides_on_device && (r = launch_mark(num_ended, ns))) return r;
            mark(6, ns);
            if (!ok(hipEventRecord(side.num_done, ns))) return fail(FB_EHIP, "lfmmi_loss_grad: event record failed");
            // the shortest range, on the numerators' stream
            if (!wait_slot(ns, 4)) return fail(FB_EHIP, "lfmmi_loss_grad: stream wait on a value failed");
            if ((r = run_posteriors(q, 2, lengths, B, N, D, grad, ns, slot_range(4), false, offs))) return r;
            // The range before it: its recursions end before the numerator launch does (which only gets the compute
            // units that finished sequences have left), so the denominator's share of its gradient does not wait for
            // the numerators, whose share a small launch adds afterwards (as in the schedule for equal lengths below).
            if (!wait_slot(gs[2], 3)) return fail(FB_EHIP, "lfmmi_loss_grad: stream wait on a value failed");
            if ((r = run_posteriors(&q[0], 1, lengths, B, N, D, grad, gs[2], slot_range(3), false, offs))) return r;
            if (!ok(hipStreamWaitEvent(gs[2], side.num_done, 0))) return fail(FB_EHIP, "lfmmi_loss_grad: stream wait failed");
            if ((r = run_posteriors(&q[1], 1, lengths, B, N, D, grad, gs[2], slot_range(3), true))) return r;
            // The second range: the numerators are done long before its recursions unless all lengths are (nearly)
            // equal.  Then no compute unit falls free before the denominator launch ends, the numerator recursions
            // only start there, and the range's gradient should not wait for them: a word written on the device when
            // the range is released says which it is, and the gradient launch takes both graphs or the denominator's
            // share alone, in which case the launch behind it adds the numerators' (same sums, same order either way).
            // (Only the gradient kernel and the kernel that adds a packed graph's share read that word.)
            if (!wait_slot(gs[1], 2)) return fail(FB_EHIP, "lfmmi_loss_grad: stream wait failed");
            if (decides_on_device) {
                int32_t *fused2 = (int32_t *)(done + kDoneFused);
                Offsets offs2 = offs, add2;
                offs2.fused = add2.fused = fused2;
                if ((r = launch_decide(num_ended, 1u, fused2, gs[1]))) return r;
                if ((r = run_posteriors(q, 2, lengths, B, N, D, grad, gs[1], slot_range(2), false, offs2))) return r;
                if (!ok(hipStreamWaitEvent(gs[1], side.num_done, 0))) return fail(FB_EHIP, "lfmmi_loss_grad: stream wait failed");
                if ((r = run_posteriors(&q[1], 1, lengths, B, N, D, grad, gs[1], slot_range(2), true, add2))) return r;
            } else {
                if (!ok(hipStreamWaitEvent(gs[1], side.num_done, 0))) return fail(FB_EHIP, "lfmmi_loss_grad: stream wait failed");
                if ((r = run_posteriors(q, 2, lengths, B, N, D, grad, gs[1], slot_range(2), false, offs))) return r;
            }
            if (part1 < cut[1]) {
                if (!wait_slot(ns, 1)) return fail(FB_EHIP, "lfmmi_loss_grad: stream wait on a value failed");
                if ((r = run_posteriors(q, 2, lengths, B, N, D, grad, ns, slot_range(1), false, offs))) return r;
            }
            if (!ok(hipStreamWaitEvent(main_s, side.num_done, 0))) return fail(FB_EHIP, "lfmmi_loss_grad: stream wait failed");
            return run_posteriors(q, 2, lengths, B, N, D, grad, main_s, RankRange{order, 0, part1}, false, offs);
        };
        rc = stages();
        for (int g = 1; g < kGroups; ++g)
            if ((!ok(hipEventRecord(side.group_done[g - 1], gs[g])) || !ok(hipStreamWaitEvent(main_s, side.group_done[g - 1], 0))) &&
                rc == FB_OK)
                rc = fail(FB_EHIP, "lfmmi_loss_grad: joining the group streams failed");
        if (rc) return rc;
        mark(3, main_s);
    } else if (in_groups && side.groups_ok && B >= 8 * kGroups) {
        // Length groups by launches: the same ranges where a stream cannot wait for a word, or while the caller's
        // stream is being captured into a graph (such a wait cannot be recorded).  Every range has a denominator
        // launch and a gradient launch of its own on a stream of its own, and the gradient of a range starts when
        // that range's launch is done.  The numerators of all sequences are one launch behind the denominator launch
        // of the last range (a few very short sequences).
        const bool fills = side.n_cu > 0 && 2 * (int64_t)B >= side.n_cu;
        const int32_t cut[kGroups + 1] = {0, group_cut(B, 0, fills), group_cut(B, 1, fills), group_cut(B, 2, fills), B};
        hipStream_t gs[kGroups] = {main_s, side.group[0], side.group[1], side.group[2]};
        auto ok = [](hipError_t e) { return e == hipSuccess; };
        mark(0, main_s);
        if ((rc = launch_order(lengths, B, N, order, done, main_s))) return rc;
        if (!ok(hipEventRecord(side.fork, main_s))) return fail(FB_EHIP, "lfmmi_loss_grad: event record failed");
        for (int g = 1; g < kGroups; ++g)
            if (!ok(hipStreamWaitEvent(gs[g], side.fork, 0))) return fail(FB_EHIP, "lfmmi_loss_grad: stream wait failed");
        mark(1, main_s);
        // From here on the side streams hold work of this call: whatever happens, the caller's stream waits
        // for them before the call returns.
        auto stages = [&]() -> int {
            int r;
            for (int g = 0; g < kGroups; ++g) {
                const RankRange range{order, cut[g], cut[g + 1] - cut[g]};
                // The workgroups of the longest range should be the first to be placed.  When calls follow one
                // another without a pause all four launches are already queued when the fork event fires and
                // would be dispatched at the same moment; an empty kernel in front of the others holds them
                // back by a launch latency (measured: 0.1 ms per call).
                if (g > 0 && (r = launch_delay(gs[g]))) return r;
                if ((r = run_recursion(den, emis, lengths, B, N, D, dd, 2, gs[g], false, range))) return r;
            }
            mark(5, gs[kGroups - 1]);
            if ((r = run_recursion(num, emis, lengths, B, N, D, dn, 2, gs[kGroups - 1], false, RankRange{order, 0, B}))) return r;
            mark(6, gs[kGroups - 1]);
            if (!ok(hipEventRecord(side.num_done, gs[kGroups - 1]))) return fail(FB_EHIP, "lfmmi_loss_grad: event record failed");
            for (int g = kGroups - 1; g >= 0; --g) {
                const RankRange range{order, cut[g], cut[g + 1] - cut[g]};
                if (g == kGroups - 2) {
                    // This range's recursions end before the numerator launch does (it only gets the compute units
                    // that short sequences have left): the denominator's share of its gradient does not wait for
                    // the numerators, whose share a small launch adds afterwards (as in the schedule for equal
                    // lengths below).
                    if ((r = run_posteriors(&q[0], 1, lengths, B, N, D, grad, gs[g], range, false, offs))) return r;
                    if (!ok(hipStreamWaitEvent(gs[g], side.num_done, 0))) return fail(FB_EHIP, "lfmmi_loss_grad: stream wait failed");
                    if ((r = run_posteriors(&q[1], 1, lengths, B, N, D, grad, gs[g], range, true))) return r;
                    continue;
                }
                if (g < kGroups - 1 && !ok(hipStreamWaitEvent(gs[g], side.num_done, 0)))
                    return fail(FB_EHIP, "lfmmi_loss_grad: stream wait failed");
                if (g == 0) mark(2, main_s);   // the longest sequences' recursions are done: the last gradient launch starts
                if ((r = run_posteriors(q, 2, lengths, B, N, D, grad, gs[g], range, false, offs))) return r;
            }
            return FB_OK;
        };
        rc = stages();
        for (int g = 1; g < kGroups; ++g)
            if ((!ok(hipEventRecord(side.group_done[g - 1], gs[g])) || !ok(hipStreamWaitEvent(main_s, side.group_done[g - 1], 0))) &&
                rc == FB_OK)
                rc = fail(FB_EHIP, "lfmmi_loss_grad: joining the group streams failed");
        if (rc) return rc;
        mark(3, main_s);
    } else if (num_apart && side.ok) {
        // Sequences of (nearly) equal length whose denominator workgroups fill the chip: no compute unit falls
        // free before the denominator recursion ends, so the numerator recursion cannot run beside it and would
        // stand between it and the gradient.  Here the denominator's share of the gradient (minus its pdf
        // posteriors, every row of the output) starts as soon as the denominator recursion is done, the numerator
        // recursion runs beside that launch, and a last small launch adds the numerators' pdf posteriors to the
        // rows (each touches only the pdfs its sequence's graph uses).
        if (hipEventRecord(side.fork, main_s) != hipSuccess || hipStreamWaitEvent(side.stream, side.fork, 0) != hipSuccess)
            return fail(FB_EHIP, "lfmmi_loss_grad: forking the side stream failed");
        mark(0, main_s);
        mark(1, main_s);
        rc = run_recursion(den, emis, lengths, B, N, D, dd, 2, main_s);
        mark(2, main_s);
        mark(5, side.stream);
        if (rc == FB_OK) rc = run_recursion(num, emis, lengths, B, N, D, dn, 2, side.stream);
        mark(6, side.stream);
        if (rc == FB_OK) rc = run_posteriors(&q[0], 1, lengths, B, N, D, grad, main_s, RankRange(), false, offs);
        // the caller's stream waits for the side stream also when a launch has failed
        if ((hipEventRecord(side.join, side.stream) != hipSuccess || hipStreamWaitEvent(main_s, side.join, 0) != hipSuccess) &&
            rc == FB_OK)
            rc = fail(FB_EHIP, "lfmmi_loss_grad: joining the side stream failed");
        if (rc) return rc;
        if ((rc = run_posteriors(&q[1], 1, lengths, B, N, D, grad, main_s, RankRange(), true))) return rc;
        mark(3, main_s);
    } else {
        // One launch per stage: the denominator launch on the caller's stream, the (much smaller) numerator
        // launch beside it on the library's side stream, then the gradient.
        const bool fork = side.ok && hipEventRecord(side.fork, main_s) == hipSuccess &&
                          hipStreamWaitEvent(side.stream, side.fork, 0) == hipSuccess;
        hipStream_t num_s = fork ? side.stream : main_s;
        mark(0, main_s);
        mark(1, main_s);
        rc = run_recursion(den, emis, lengths, B, N, D, dd, 2, main_s);
        mark(2, main_s);
        mark(5, num_s);
        if (rc == FB_OK) rc = run_recursion(num, emis, lengths, B, N, D, dn, 2, num_s);
        mark(6, num_s);
        // the caller's stream waits for the side stream also when a launch has failed
        if (fork && (hipEventRecord(side.join, side.stream) != hipSuccess || hipStreamWaitEvent(main_s, side.join, 0) != hipSuccess) &&
            rc == FB_OK)
            rc = fail(FB_EHIP, "lfmmi_loss_grad: joining the side stream failed");
        if (rc) return rc;
        if (fork) mark(2, main_s);   // the gradient stage starts when both recursion launches are done
        if ((rc = run_posteriors(q, 2, lengths, B, N, D, grad, stream, RankRange(), false, offs))) return rc;
        mark(3, main_s);
    }
    rc = launch_loss(zn, zd, lengths, B, loss, stream);
    mark(4, main_s);
    if (g_prof.on && rc == FB_OK) g_prof.recorded = true;
    return rc;
}

int lfmmi_loss_grad(const fb_graph *den, const fb_graph *num, const float *emis, const int32_t *lengths, int32_t B,
                    int32_t N, int32_t D, double *loss, double *logz_num, double *logz_den, float *grad, void *ws,
                    size_t ws_bytes, fb_stream stream)
{
    // Without a host copy of the lengths nothing is known about them here; the schedule in length groups needs only
    // ranks, which the device computes, and costs little when the lengths turn out to be equal.
    return lfmmi_run(den, num, emis, lengths, B, N, D, loss, logz_num, logz_den, grad, ws, ws_bytes, stream, true, false);
}

size_t fb_static_scratch_bytes(void) { return kStaticScratchBytes; }

int lfmmi_loss_grad_static(const fb_graph *den, const fb_graph *num, const float *emis, const int32_t *lengths, int32_t B,
                           int32_t N, int32_t D, double *loss, double *logz_num, double *logz_den, float *grad,
                           fb_stream stream)
{
    int rc = check_common("lfmmi_loss_grad_static", den, emis, lengths, B, N, D);
    if (rc) return rc;
    if ((rc = check_common("lfmmi_loss_grad_static", num, emis, lengths, B, N, D))) return rc;
    const size_t need = fb_lfmmi_workspace_bytes(den, num, B, N, D);
    if (need == 0) return fail(FB_EINVAL, "lfmmi_loss_grad_static: these graphs and sizes have no workspace size");
    if (need > kStaticScratchBytes)
        return fail(FB_EUNSUPPORTED, "lfmmi_loss_grad_static: the call needs " + std::to_string(need) +
                                         " bytes of workspace, the built-in scratch memory holds " +
                                         std::to_string(kStaticScratchBytes) + " (use lfmmi_loss_grad with a workspace)");
    void *ws = static_scratch();
    if (!ws) return FB_EHIP;
    // (every word of the workspace that a kernel reads is written earlier in the same call: nothing to clear)
    return lfmmi_run(den, num, emis, lengths, B, N, D, loss, logz_num, logz_den, grad, ws, kStaticScratchBytes, stream, true, false);
}

int lfmmi_loss_grad_ragged(const fb_graph *den, const fb_graph *num, const float *emis, const int32_t *lengths,
                           const int32_t *lengths_host, int32_t B, int32_t N, int32_t D, double *loss, double *logz_num,
                           double *logz_den, float *grad, void *ws, size_t ws_bytes, fb_stream stream)
{
    // Length groups pay when compute units would otherwise idle: the shorter sequences leave
    // (1 - mean length / longest length) of the denominator launch's compute-unit time unused.
    bool in_groups = false, num_apart = false;
    if (lengths_host && B > 0 && N > 0) {
        int64_t sum = 0;
        int32_t longest = 0;
        for (int32_t b = 0; b < B; ++b) {
            const int32_t l = std::min(std::max(lengths_host[b], 0), N);
            sum += l;
            longest = std::max(longest, l);
        }
        in_groups = longest > 0 && (double)sum < 0.85 * (double)longest * B;
        // Otherwise, when the denominator workgroups (two per sequence, each filling a compute unit) take the
        // whole chip, the numerators' share of the gradient goes apart (see lfmmi_run).
        const int n_cu = side_stream().n_cu;
        num_apart = !in_groups && longest > 0 && den && den->nw == kNWShared && n_cu > 0 && 2 * (int64_t)B >= n_cu;
    }
    return lfmmi_run(den, num, emis, lengths, B, N, D, loss, logz_num, logz_den, grad, ws, ws_bytes, stream, in_groups, num_apart);
}

}  // extern "C"
