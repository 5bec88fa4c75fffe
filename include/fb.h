/*
 * fb.h -- C ABI of the MI355X forward-backward / LF-MMI library (libfb_amd.so).
 *
 * The library computes, on one gfx950 GPU and in the log semifield of the
 * paper (Semiring-algebra section, Eq. 8-12: a (+) b = log(e^a + e^b),
 * a (x) b = a + b, zero = -inf, one = 0):
 *
 *   fb_alpha         alpha_n = v_n o (T^t alpha_{n-1})                 Eq. 13
 *   fb_beta          beta_n  = T (beta_{n+1} o v_{n+1})                Eq. 14
 *   fb_posteriors    p(z_n | x) = alpha_n beta_n / sum_z alpha_N(z)    Eq. 15
 *   lfmmi_loss_grad  L = log p(X|G_num) - log p(X|G_den), dL/dphi      Eq. 16-17
 *   lfmmi_loss_grad_ragged  the same, scheduled for sequences of unequal length
 *
 * and, with the tropical semiring ((+) = max) in place of the log semiring,
 *
 *   fb_viterbi       best-path score and a path that attains it        Conclusion section
 *
 * for a batch of sequences (Dealing-with-batches section).  All logs are
 * natural.  Frames and states are numbered from 0.
 *
 * Model.  A graph has K states and E arcs (src -> dst, log-weight logw); only
 * arcs that are not the semiring zero are stored.  State k emits through pdf
 * pdf[k] in [0, D): v_n[k] = emis[b][n][pdf[k]].  alpha_0 = init (x) v_0 (the
 * first state emits the first frame, so T frames use T-1 arcs),
 * beta_{T-1} = final, log Z = (+)-sum_k alpha_{T-1}[k] (x) final[k].
 * -inf is a legal value of init, final, logw and emis; NaN and +inf are not.
 * Parallel arcs are kept apart (their weights (+)-add).
 *
 * Two kinds of graph:
 *   shared  one graph used by every sequence of the batch (the denominator
 *           graph; the paper replicates it on the block diagonal, here it is
 *           stored once);
 *   packed  n_seq graphs concatenated block-diagonally, sequence b owning the
 *           states [state_off[b], state_off[b+1]) (numerator graphs).
 *
 * Pointers.  Unless a comment says "host", every array argument of a compute
 * call is a DEVICE pointer owned by the caller; the library neither allocates
 * nor frees nor synchronises in a compute call, it only enqueues kernels on
 * `stream` (a hipStream_t, NULL = the default stream).  Inputs are read-only.
 * Outputs are overwritten in full unless stated.  A compute call may be recorded
 * into a HIP graph by stream capture on `stream` (streams of the library's own
 * that a call uses are forked from and joined into `stream` with events; nothing
 * is cleared with a memset; the one step that cannot be recorded, a stream wait
 * on a value in the LF-MMI calls, is replaced by waits on events while `stream` is
 * capturing).
 *
 * Layouts (row-major, last index fastest):
 *   emis, pdf_post, grad   float [B][N][D]
 *   lengths                int32 [B]; sequence b has lengths[b] real frames,
 *                          the rest of its N frames is padding and is ignored.
 *                          A length is clamped to [0, N]; a sequence of length
 *                          0 is skipped (log Z = -inf, zero posteriors, no
 *                          contribution to the loss).
 *   alpha, beta, state_post
 *       shared graph       float [B][N][K]
 *       packed graphs      float [N][K]   (K = all states of all sequences;
 *                                          sequence b fills its own columns)
 *   alpha_cum, beta_cum    double [B][N]
 *   logz                   double [B]
 *
 * Normalised storage.  Stored alpha/beta rows are shifted so that single
 * precision keeps its resolution on long sequences:
 *   true alpha_n[k] = alpha[..n..][k] + alpha_cum[b][n]
 *   true beta_n[k]  = beta[..n..][k]  + beta_cum[b][n]
 * (the shift of frame n, accumulated in double over the frames the recursion has passed: from
 * the first frame for alpha, from the last for beta).  The shifts cancel in Eq. 15, so
 * posteriors do not depend on them.  Rows of padded frames hold -inf (alpha, beta) or 0
 * (shifts, posteriors, grad).
 *
 * Precision.  Exponentials and logarithms are single precision everywhere.
 * The normalised state vector of the recursions is carried either in single or
 * in double precision.  A single-precision log value x carries a rounding error
 * of about 3e-8 * |x| per time step, so single carriers are accurate when the
 * states that matter for the posterior lie within a few tens of the frame's
 * best state (densely connected graphs such as the denominator); in long
 * left-to-right chains a state can matter while its alpha is far below the
 * frame's best, and double carriers keep the 1e-5 posterior accuracy there.
 * The alpha / beta arrays of fb_alpha / fb_beta are float in both cases.
 *
 * Errors.  Every call returns FB_OK (0) or a negative code and never throws;
 * fb_last_error() gives a thread-local description of the last failure.
 * Kernel launches are asynchronous: an error inside a kernel surfaces at the
 * caller's next synchronisation.  A sequence with no complete path has
 * log Z = -inf and zero posteriors / gradient -- that is not an error.
 */
#ifndef FB_AMD_H
#define FB_AMD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fb_graph fb_graph; /* opaque; owns host and device copies of its layouts */
typedef void *fb_stream;          /* hipStream_t */

enum {
    FB_OK = 0,
    FB_EINVAL = -1,      /* malformed argument (see each call)                       */
    FB_ENOMEM = -2,      /* host or device allocation failed                         */
    FB_EHIP = -3,        /* a HIP runtime call failed (no device, launch error, ...) */
    FB_EUNSUPPORTED = -4 /* valid input beyond a documented limit of the kernels     */
};

/* fb_graph_create flags */
enum {
    FB_GRAPH_HOST_ONLY = 1, /* build and keep the layouts on the host only: no GPU is touched;
                               the handle serves fb_graph_layout* but no compute call */
    FB_GRAPH_WIDE_STATE = 2, /* carry the state vectors in double (see "Precision" below) */
    FB_GRAPH_NARROW_STATE = 4 /* carry them in single; with neither flag the library chooses:
                               double for small (sub-)graphs (< 4096 arcs and <= 1024 states each),
                               single otherwise.  Single precision on long left-to-right chains (the
                               numerator graphs) does NOT meet the 1e-5 posterior tolerance: a state
                               can matter while its alpha lies thousands below the frame's best, where
                               a float log value is spaced 2e-4 apart (1.2e-5 measured on chains of
                               150 phones); use it only where that is acceptable */
};

/* Arrays that fb_graph_layout can copy out (graph-layout step; integer work, one
 * well-defined answer).  "in" = arcs stably sorted by destination (what T^t of
 * Eq. 13 gathers), "out" = arcs stably sorted by source (T of Eq. 14); "stable"
 * = ties keep ascending original arc index.  *_PERM[i] is the original index
 * of the i-th sorted arc; *_W the weights permuted, never altered. */
enum {
    FB_IN_PTR = 0,     /* int32 [K+1]  arcs entering state j are IN_*[ptr[j] .. ptr[j+1])  */
    FB_IN_SRC = 1,     /* int32 [E]                                                          */
    FB_IN_W = 2,       /* float [E]                                                          */
    FB_IN_PERM = 3,    /* int32 [E]                                                          */
    FB_OUT_PTR = 4,    /* int32 [K+1]  arcs leaving state i are OUT_*[ptr[i] .. ptr[i+1])   */
    FB_OUT_DST = 5,    /* int32 [E]                                                          */
    FB_OUT_W = 6,      /* float [E]                                                          */
    FB_OUT_PERM = 7,   /* int32 [E]                                                          */
    FB_PDF_PTR = 8,    /* int32 [D+1]  states tied to pdf d are PDF_STATES[ptr[d] .. ptr[d+1]) */
    FB_PDF_STATES = 9  /* int32 [K]    states stably sorted by pdf id                        */
};

/*
 * Build a graph (graph-layout step; Matrix-based-implementation section: T[i][j]
 * is the weight of arc i -> j, stored sparsely).
 *   src, dst, logw  host, [E], arcs in any order
 *   pdf, init, final host, [K]
 *   D               number of pdfs (columns of emis)
 *   n_seq, state_off  n_seq = 0 and NULL: shared graph.  n_seq = B > 0 and host
 *                   int32 [B+1]: packed graphs, state_off[0] = 0, non-decreasing,
 *                   state_off[B] = K, every graph non-empty.
 * The arrays are copied; the caller may free them on return.
 * FB_EINVAL: NULL pointer, K <= 0, E < 0, D <= 0, an arc endpoint outside [0,K),
 *   a pdf id outside [0,D), a NaN or +inf weight / init / final, bad state_off,
 *   an arc joining two packed graphs.  FB_EUNSUPPORTED: a (sub-)graph too large
 *   for the on-chip state vector (see fb_limits).  FB_EHIP / FB_ENOMEM: upload failed.
 */
int fb_graph_create(fb_graph **out, int32_t K, int64_t E, const int32_t *src, const int32_t *dst,
                    const float *logw, const int32_t *pdf, const float *init, const float *final_,
                    int32_t D, int32_t n_seq, const int32_t *state_off, uint32_t flags);

/* Free a graph and its device memory.  NULL is allowed.  The caller must have
 * synchronised every stream that still uses it. */
int fb_graph_destroy(fb_graph *g);

/* Number of elements of layout array `which`, or a negative error code. */
int64_t fb_graph_layout_size(const fb_graph *g, int which);

/* Copy layout array `which` to host_out (host pointer); bytes must be exactly
 * 4 * fb_graph_layout_size().  FB_EINVAL otherwise. */
int fb_graph_layout(const fb_graph *g, int which, void *host_out, size_t bytes);

/*
 * Diagnostic, host only: apply the static work plan the kernels walk for this
 * graph, on the host and in double precision, to a vector x (host).
 *   which = 0  forward plan:  y[j] = (+)-sum over arcs entering j of (w (x) x[src]), log2 units
 *   which = 1  backward plan: y[i] = (+)-sum over arcs leaving i of (w (x) x[dst]), log2 units
 *   which = 2  pdf plan:      y[d] = sum of x over the states tied to pdf d (ordinary sum)
 *   which = 5, 6  the forward / backward plan of the probability-domain kernel (fb_graph_linear_weights = 2, also
 *              kept by host-only handles of graphs that qualify), in ordinary arithmetic:
 *              y[j] = sum over arcs entering (leaving) j of e^logw x[src] - x and y are plain numbers here;
 *              FB_EUNSUPPORTED if the graph has no such plan
 *   which = 3, 4  the forward / backward plan in the form with weights as 2^w (see
 *              fb_graph_linear_weights), whatever form the device copy has: same results to
 *              rounding; FB_EUNSUPPORTED if a weight of the graph is out of that form's range;
 *              the walk also checks what the multiplying kernel relies on (an internal
 *              error, FB_EHIP, if it does not hold)
 * sub: 0 for a shared graph, the sequence index for packed graphs; x and y use
 * the sub-graph's local state numbering (y: pdf ids for which = 2; entries
 * without a row keep their value).  Weights are the graph's log-weights times
 * log2(e), rounded to float.  Lets a CPU-only test check the scheduling logic.
 */
int fb_graph_schedule_apply_host(const fb_graph *g, int which, int32_t sub, const double *x, double *y);

/* Host-side check of a host copy of lengths: FB_EINVAL if NULL, B <= 0, N <= 0
 * or any length is outside [1, N].  (The compute calls themselves only see the
 * device copy and clamp.) */
int fb_check_lengths(const int32_t *lengths_host, int32_t B, int32_t N);

/*
 * Forward recursion, Eq. 13, for every sequence of the batch.
 *   alpha      out, nullable (then only the shifts and log Z are produced)
 *   alpha_cum  out, double [B][N], nullable
 *   logz       out, double [B], nullable: log Z_b = (+)-sum_k alpha_{T-1}[k] (x) final[k]
 * FB_EINVAL: g NULL or host-only, emis / lengths NULL, B/N/D <= 0, D != the graph's D,
 *   packed graph with B != n_seq.  FB_EUNSUPPORTED: K and D together exceed the
 *   on-chip memory of a compute unit (fb_limits).
 */
int fb_alpha(const fb_graph *g, const float *emis, const int32_t *lengths, int32_t B, int32_t N, int32_t D,
             float *alpha, double *alpha_cum, double *logz, fb_stream stream);

/*
 * Backward recursion, Eq. 14 (with v_{n+1}, as in the scalar Eq. 3).
 *   beta, beta_cum  out, nullable, as for fb_alpha
 *   logz            out, nullable: log Z_b evaluated at the first frame,
 *                   (+)-sum_k init[k] (x) v_0[k] (x) beta_0[k]; equals fb_alpha's up to rounding
 * Errors as fb_alpha.
 */
int fb_beta(const fb_graph *g, const float *emis, const int32_t *lengths, int32_t B, int32_t N, int32_t D,
            float *beta, double *beta_cum, double *logz, fb_stream stream);

/*
 * State and pdf posteriors, Eq. 15, from the normalised alpha and beta of
 * fb_alpha / fb_beta (the offsets are not needed: they cancel).
 *   state_post  out, nullable: gamma[.][n][k] = exp(alpha_n[k] (x) beta_n[k] (/) log Z)
 *   pdf_post    out, nullable: rho[b][n][d] = sum of gamma over the states tied to pdf d
 * The normaliser is evaluated on each frame as (+)-sum_k alpha_n[k] (x) beta_n[k],
 * which equals log Z for every n, so rounding accumulated along the recursion
 * cancels.  Padded frames get 0.  Errors as fb_alpha (alpha, beta, lengths must
 * not be NULL; at least one output must be given).
 */
int fb_posteriors(const fb_graph *g, const float *alpha, const float *beta, const int32_t *lengths,
                  int32_t B, int32_t N, int32_t D, float *state_post, float *pdf_post, fb_stream stream);

/* Bytes of device workspace lfmmi_loss_grad needs for these sizes (0 on bad arguments). */
size_t fb_lfmmi_workspace_bytes(const fb_graph *den, const fb_graph *num, int32_t B, int32_t N, int32_t D);

/*
 * LF-MMI objective and its derivative w.r.t. the network output (Eq. 16-17):
 *   loss  = sum_b ( log Z_num[b] - log Z_den[b] )          (no sign flip, no averaging)
 *   grad[b][n][d] = rho_num[b][n][d] - rho_den[b][n][d]    (0 on padded frames)
 *   den   shared graph, num packed graphs with n_seq = B, both built with this D
 *   loss  out, device double [1]; logz_num, logz_den out, device double [B], nullable
 *   ws    device scratch of at least fb_lfmmi_workspace_bytes(), 256-byte aligned;
 *         its contents are undefined before and after the call
 * Schedule.  For B >= 32 the batch is worked in order of length (the order is computed on
 * the device from `lengths`; no host copy of the lengths is needed).  The denominator
 * recursions of all sequences are one launch, longest sequences first; the ranks are cut
 * into ranges, each with a progress counter its recursion workgroups increment when they
 * are done, and every range has a gradient launch of its own, on the caller's stream and
 * three of the library's, that waits for its counter (hipStreamWaitValue32) and runs on the
 * compute units its sequences have left while the longest recursions are still going.  The
 * numerator launch runs on one of those streams once the denominator workgroups hold their
 * compute units.  Where the device cannot wait for a word, or while `stream` is being
 * captured, every range has a denominator launch of its own instead and the waits are on
 * events.  For B < 32 there is one launch per stage, the numerator launch on a stream of
 * the library's beside the denominator launch.  The library's streams are forked from
 * `stream` and joined back into it with events, so for the caller everything is ordered on
 * `stream` as usual.  FB_AMD_SERIAL=1 in the environment keeps all launches on `stream`;
 * FB_AMD_GROUPS=0 creates only one of the library's streams (with the caller's, the four
 * take the hardware queues a process has) and so keeps to one launch per stage.  Those
 * streams, their events and the stage timer belong to the process; a lock is held while a call
 * enqueues its work, so LF-MMI calls from several host threads are safe and their work is
 * ordered on the library's streams in the order of the calls (each call still uses only its
 * own workspace and outputs).
 * FB_EINVAL: as fb_alpha, or ws too small / NULL, den packed, num shared.
 */
int lfmmi_loss_grad(const fb_graph *den, const fb_graph *num, const float *emis, const int32_t *lengths,
                    int32_t B, int32_t N, int32_t D, double *loss, double *logz_num, double *logz_den,
                    float *grad, void *ws, size_t ws_bytes, fb_stream stream);

/*
 * The same objective and derivative (Eq. 16-17), given a host copy of the lengths:
 *   lengths_host  host int32 [B], the values of `lengths`; used to decide how the work is
 *                 scheduled, never for the results (if it disagrees with `lengths` the call is
 *                 still correct, only possibly slower); NULL: exactly lfmmi_loss_grad
 * What the lengths decide: sequences that differ in length (the shorter ones would leave more
 * than 15 % of the denominator recursion's compute-unit time idle) are scheduled as in
 * lfmmi_loss_grad.  For sequences of (nearly) equal length, a denominator graph large enough
 * for the 16-wave kernel and 2 B >= the number of compute units, no compute unit falls free
 * before the denominator recursion ends: then there is one denominator launch, the
 * denominator's share of the gradient is formed while the numerator recursion runs on the
 * library's side stream, and the numerators' share is added by a last small launch - the same
 * as lfmmi_loss_grad reaches with its counters, without them (so also under stream capture).
 * Otherwise one launch per stage.  Same arguments, workspace and errors as lfmmi_loss_grad,
 * same loss and log Z bit for bit, the same gradient to rounding (the launches of the
 * schedules form the same sums in different orders).
 */
int lfmmi_loss_grad_ragged(const fb_graph *den, const fb_graph *num, const float *emis, const int32_t *lengths,
                           const int32_t *lengths_host, int32_t B, int32_t N, int32_t D, double *loss,
                           double *logz_num, double *logz_den, float *grad, void *ws, size_t ws_bytes,
                           fb_stream stream);

/*
 * lfmmi_loss_grad for callers that cannot allocate device memory or have none to spare for a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same results as lfmmi_loss_grad (same kernels, same schedule); the workspace is
 * scratch memory built into the library's image, fb_static_scratch_bytes() = 16 MiB on every
 * GPU the library runs on, held until the process ends.  The call allocates nothing and frees
 * nothing (the address of the memory on a device is looked up when the first graph is created
 * on it, else at the first call).
 *   loss, logz_num, logz_den, grad   as in lfmmi_loss_grad, caller-owned device memory
 * Sizes whose fb_lfmmi_workspace_bytes() exceeds fb_static_scratch_bytes() are refused with
 * FB_EUNSUPPORTED (the message gives both figures); other errors as lfmmi_loss_grad.
 * Every call on a GPU shares that GPU's scratch memory, which keeps the last call's contents
 * (a call writes every word it reads, so nothing has to be cleared): calls that overlap on
 * one GPU, on whatever streams, race with each other.
 */
int lfmmi_loss_grad_static(const fb_graph *den, const fb_graph *num, const float *emis, const int32_t *lengths,
                           int32_t B, int32_t N, int32_t D, double *loss, double *logz_num, double *logz_den,
                           float *grad, fb_stream stream);

/* Bytes of the scratch memory lfmmi_loss_grad_static works in. */
size_t fb_static_scratch_bytes(void);

/* Bytes of device workspace fb_viterbi needs for these sizes (0 on bad arguments). */
size_t fb_viterbi_workspace_bytes(const fb_graph *g, int32_t B, int32_t N);

/*
 * Best path (Conclusion section: the same forward recursion with the log semiring
 * replaced by the tropical semiring, (+) = max, is the Viterbi algorithm):
 *   delta_0[k] = init[k] + v_0[k];  delta_n[j] = v_n[j] + max_{arcs e into j} ( w_e + delta_{n-1}[src_e] )
 *   score[b]   = max_k ( delta_{N_b - 1}[k] + final[k] )
 *   path[b][n] = the state (global numbering) at frame n of a path that attains the score,
 *                for n < lengths[b]; -1 on padded frames and when the score is -inf.
 * Several paths may attain the score; which one is returned is fixed for a given graph and
 * input (results do not depend on timing) but otherwise unspecified.
 *   score  out, device double [B];  path  out, device int32 [B][N]
 *   ws     device scratch of at least fb_viterbi_workspace_bytes(), 256-byte aligned
 *          (the back-pointers: 2 bytes per state and frame, a little more for graphs with very long rows)
 * Errors as fb_alpha.
 */
int fb_viterbi(const fb_graph *g, const float *emis, const int32_t *lengths, int32_t B, int32_t N, int32_t D,
               double *score, int32_t *path, void *ws, size_t ws_bytes, fb_stream stream);

/*
 * Comparison mode: the "leaky-HMM" denominator (Python and Julia recipes section and Table 1: the approximation the
 * paper's comparison system makes, in the probability domain with a scale per frame).  The paper defines it only
 * by reference; it is taken here as a model with a plain definition: before every transition a fraction `leak` of
 * the total probability is handed out again over the states in proportion to pi = exp(init) / sum exp(init), i.e.
 * the hidden Markov model with the transition matrix T' = (I + leak 1 pi^T) T and the graph's own initial and
 * final weights.  log Z and the pdf posteriors (Eq. 13-15 for T') of every sequence, in one call; leak = 0 gives
 * the graph itself.  Not part of lfmmi_loss_grad, and not tuned like it: a plain kernel, one workgroup per sequence.
 * Vectors are float, rescaled to sum 1 in every frame, with no fallback: an entry below 2^-126 of its frame's total
 * is taken as 0 (as in any implementation of this kind; harmless unless a later frame's emissions lift such a state
 * by as much again, which takes emissions that differ by more than 87 nats between live states of one frame).
 *   g         a shared graph (n_seq == 0)
 *   emis      device float [B][N][D];  lengths  device int32 [B]
 *   leak      in [0, 1]
 *   logz      out, device double [B] (-inf for a sequence without a path, whose posteriors are 0)
 *   pdf_post  out, device float [B][N][D], 0 on padded frames
 *   ws        device scratch of at least fb_leaky_workspace_bytes() (the forward vectors: 4 bytes per state and frame)
 * FB_EINVAL: NULL arguments, a packed or host-only graph, sizes <= 0, D != the graph's D, leak outside [0, 1],
 * workspace missing or too small.  FB_EUNSUPPORTED: more than 8192 states, or four state vectors and an emission row
 * exceed the 160 KB of on-chip memory of a compute unit (16 K + 4 D bytes).
 */
size_t fb_leaky_workspace_bytes(const fb_graph *g, int32_t B, int32_t N);
int fb_leaky_posteriors(const fb_graph *g, const float *emis, const int32_t *lengths, int32_t B, int32_t N, int32_t D,
                        float leak, double *logz, float *pdf_post, void *ws, size_t ws_bytes, fb_stream stream);

/* Limits of the kernels for a graph / batch shape: the largest number of states
 * one (sub-)graph may have so that its state vectors and one emission row of D
 * pdfs fit in the 160 KB of on-chip memory of a gfx950 compute unit.
 * shared != 0: shared-graph kernels; 0: packed-graph kernels. */
int32_t fb_limits_max_states(int32_t D, int shared);

/* Diagnostic: which form of the arc weights the graph's device plans carry.  1: 2^w, for the
 * kernel instantiation that multiplies (large graphs with float vectors whose finite weights
 * all lie within 64 binary orders of magnitude of 1: there the product form is exact to
 * rounding); 0: w, added in the exponent (every other graph, and every graph when
 * FB_AMD_LINEAR=0 is in the environment); -1: g is NULL.  The results of the compute calls are
 * the same to rounding either way. */
int fb_graph_linear_weights(const fb_graph *g);

/* Diagnostic: how many (sequence, direction) runs the probability-domain recursion kernel has given up and
 * redone in the log form since the library was loaded (see fb_graph_linear_weights: form 2).  Synchronises
 * the device. */
int64_t fb_debug_linear_restarts(void);

/* Diagnostic, host only: the cycles the gathers of one time step of the probability-domain kernel take in the
 * on-chip memory under the bank model its arc order is chosen by (32 banks of 4 bytes; a 64-lane gather is served
 * as two halves, each in as many cycles as its busiest bank has distinct addresses), and the least any order could
 * take (two cycles per gather).  backward: 0 the forward plan, 1 the backward plan.  FB_EUNSUPPORTED if the graph
 * has no such plan. */
int fb_graph_plan_cycles(const fb_graph *g, int backward, int64_t *cycles, int64_t *cycles_floor);

/*
 * Stage timing of lfmmi_loss_grad, for benchmarks.  fb_profile_enable(1) creates
 * seven HIP events (the only allocation; not allowed while a stream is being
 * captured); while enabled, lfmmi_loss_grad records one before and after each of
 * its four kernel launches, on the stream the launch goes to.  fb_profile_read
 * waits for the last recorded events and returns the milliseconds of the latest
 * call's stages: ms[0] numerator recursions (they run beside the denominator's),
 * ms[1] denominator recursions, ms[2] posteriors and gradient, ms[3] objective.  FB_EINVAL if profiling is off, ms is NULL (host
 * pointer) or no call was recorded.  fb_profile_enable(0) destroys the events.
 */
int fb_profile_enable(int on);
int fb_profile_read(float *ms);

const char *fb_strerror(int code);
const char *fb_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FB_AMD_H */
