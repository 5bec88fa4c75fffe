// The "leaky-HMM" denominator as a comparison mode (Python and Julia recipes section; Analysis section, Table 1:
// the approximation the paper's comparison system makes, in the probability domain with a scale per frame).
//
// The paper defines it only by reference.  The reading built here is a model with a plain definition: before every
// transition a fraction `leak` of the total probability is handed out again over the states in proportion to
// pi = exp(init) / sum exp(init), i.e. the hidden Markov model with the transition matrix
//     T' = (I + leak 1 pi^T) T
// and the graph's own initial and final weights.  Its forward and backward variables, log Z and posteriors are those
// of Eq. 13-15 for T'; the rank-one term is kept apart from the sparse one:
//     alpha_n = v_n o T^T (alpha_{n-1} + leak sum(alpha_{n-1}) pi)
//     beta_n  = y + leak (pi . y) 1,   y = T (v_{n+1} o beta_{n+1})
// One workgroup of 16 waves per sequence runs the forward sweep (every vector rescaled to sum 1, the logarithms of
// the scales added up in double; the vectors go to the workspace), then the backward sweep, which forms each
// frame's posteriors alpha_n o beta_n, normalised by their own sum, and adds them up per pdf in a fixed order.
// Vectors are float in LDS.  The sparse products walk plain row lists in global memory (they stay in L2): rows of
// more than 64 arcs in pieces of 256 arcs by a wave each (their sums added in order afterwards), the others one per
// thread, sorted by length in blocks of 1024 rows with the arcs of a block stored slot by slot, so that the threads
// of a wave read neighbouring words.  There is no range guard and no fallback to logarithms: an entry below 2^-126 of
// its frame's total is flushed to zero, which is this kind of method's own approximation (the exact path gives such
// a sequence up and redoes it in the log form).  This is a simple kernel for comparison, not tuned like the exact path: no
// arcs in registers, several barriers per frame, 8 bytes from L2 per arc and frame.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <numeric>
#include <string>
#include <vector>

#include "../../include/fb.h"
#include "fb_internal.h"

namespace fb {

constexpr int kLeakyThreads = 1024, kLeakyWaves = kLeakyThreads / 64;
constexpr int kLeakyLong = 64;   // rows with more arcs than this are walked by whole waves,
constexpr int kLeakyPiece = 256;  // in pieces of at most this many arcs (four per lane, all loads in flight at once)

struct LeakyDir {
    // rows of more than kLeakyLong arcs: row ids, the range of pieces of each, the arc range of each piece, arcs
    int32_t n_long, n_piece;
    const int32_t *long_row, *long_piece, *piece_ptr, *long_src;
    const float *long_w;
    // the others, in blocks of kLeakyThreads rows sorted by length: row id per place (-1: none), per block its
    // number of slots and the offset of its first slot; slot s of place t of block j is entry off[j] + s * 1024 + t
    int32_t n_block;
    const int32_t *short_row, *block_slots;
    const int64_t *block_off;
    const int32_t *ell_src;
    const float *ell_w;
};

struct LeakyDev {
    LeakyDir fwd, bwd;           // rows = destinations (arcs by source index) / rows = sources
    const float *pi, *initp, *finalp;
    const int32_t *pdf, *pdf_ptr, *pos;   // pos[k]: the place of state k among the states in pdf order
};

struct LeakyParams {
    LeakyDev G;
    const float *emis;
    const int32_t *lengths;
    int32_t B, N, D, K;
    float leak;
    double *logz;
    float *pdf_post;
    float *rows;                 // workspace [B][N][K]: the forward vectors, each with sum 1
};

namespace {

template <class T>
int up(fb_graph *g, const std::vector<T> &h, const T **dev)
{
    *dev = nullptr;
    std::vector<T> one(1);
    const std::vector<T> &src = h.empty() ? one : h;   // (a pointer the kernel may form addresses from, even if it reads nothing)
    void *p = nullptr;
    hipError_t e = hipMalloc(&p, src.size() * sizeof(T));
    if (e != hipSuccess)
        return fail(e == hipErrorOutOfMemory ? FB_ENOMEM : FB_EHIP, std::string("hipMalloc: ") + hipGetErrorString(e));
    g->allocs.push_back(p);
    e = hipMemcpy(p, src.data(), src.size() * sizeof(T), hipMemcpyHostToDevice);
    if (e != hipSuccess) return fail(FB_EHIP, std::string("hipMemcpy: ") + hipGetErrorString(e));
    *dev = (const T *)p;
    return FB_OK;
}

// rows given as ptr / col / log weight (CSR by the row index) -> the two lists of a direction
int build_dir(fb_graph *g, int32_t K, const std::vector<int32_t> &ptr, const std::vector<int32_t> &col,
              const std::vector<float> &logw, LeakyDir &d)
{
    std::vector<int32_t> order((size_t)K);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return ptr[a + 1] - ptr[a] > ptr[b + 1] - ptr[b]; });
    std::vector<int32_t> long_row, long_piece{0}, piece_ptr{0}, long_src, short_row, block_slots, ell_src;
    std::vector<float> long_w, ell_w;
    std::vector<int64_t> block_off;
    int32_t n_long = 0;
    while (n_long < K && ptr[order[n_long] + 1] - ptr[order[n_long]] > kLeakyLong) ++n_long;
    for (int32_t i = 0; i < n_long; ++i) {
        const int32_t r = order[i];
        long_row.push_back(r);
        for (int32_t e = ptr[r], n = 0; e < ptr[r + 1]; ++e, ++n) {
            if (col[e] < 0 || col[e] >= K) return fail(FB_EHIP, "internal error: leaky-HMM row list out of bounds");
            if (n > 0 && n % kLeakyPiece == 0) piece_ptr.push_back((int32_t)long_src.size());
            long_src.push_back(col[e]);
            long_w.push_back(std::exp(logw[e]));
        }
        piece_ptr.push_back((int32_t)long_src.size());
        long_piece.push_back((int32_t)piece_ptr.size() - 1);
    }
    const int32_t n_short = K - n_long;
    const int32_t n_block = (n_short + kLeakyThreads - 1) / kLeakyThreads;
    short_row.assign((size_t)n_block * kLeakyThreads, -1);
    for (int32_t j = 0; j < n_block; ++j) {
        const int32_t first = n_long + j * kLeakyThreads;
        // the block's longest row comes first; slots come in fours (the kernel loads four at a time), empty ones weigh 0
        const int32_t slots = (ptr[order[first] + 1] - ptr[order[first]] + 3) & ~3;
        block_slots.push_back(slots);
        block_off.push_back((int64_t)ell_src.size());
        ell_src.resize(ell_src.size() + (size_t)slots * kLeakyThreads, 0);
        ell_w.resize(ell_w.size() + (size_t)slots * kLeakyThreads, 0.0f);
        for (int32_t t = 0; t < kLeakyThreads && first + t < K; ++t) {
            const int32_t r = order[first + t];
            short_row[(size_t)j * kLeakyThreads + t] = r;
            for (int32_t e = ptr[r], s = 0; e < ptr[r + 1]; ++e, ++s) {
                if (s >= slots || col[e] < 0 || col[e] >= K) return fail(FB_EHIP, "internal error: leaky-HMM row list out of bounds");
                ell_src[(size_t)block_off.back() + (size_t)s * kLeakyThreads + t] = col[e];
                ell_w[(size_t)block_off.back() + (size_t)s * kLeakyThreads + t] = std::exp(logw[e]);
            }
        }
    }
    d.n_long = n_long;
    d.n_piece = (int32_t)piece_ptr.size() - 1;
    d.n_block = n_block;
    int rc;
    if ((rc = up(g, long_row, &d.long_row)) || (rc = up(g, long_piece, &d.long_piece)) || (rc = up(g, piece_ptr, &d.piece_ptr)) ||
        (rc = up(g, long_src, &d.long_src)) ||
        (rc = up(g, long_w, &d.long_w)) || (rc = up(g, short_row, &d.short_row)) || (rc = up(g, block_slots, &d.block_slots)) ||
        (rc = up(g, block_off, &d.block_off)) || (rc = up(g, ell_src, &d.ell_src)) || (rc = up(g, ell_w, &d.ell_w)))
        return rc;
    return FB_OK;
}

__device__ __forceinline__ float wsum(float v)   // a fixed tree: results do not depend on timing
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wmaxf(float v)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// sum (or maximum) over the workgroup of one value per thread; every thread gets it.  red: 2 x 16 floats, the halves
// used in turn so that a call never overwrites what a slower wave still reads from the call before.
template <bool MAX>
__device__ __forceinline__ float block_reduce(float v, float *red, int &turn)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    v = MAX ? wmaxf(v) : wsum(v);
    float *r = red + (turn & 1) * kLeakyWaves;
    ++turn;
    if (lane == 0) r[wave] = v;
    __syncthreads();
    float t = r[0];
#pragma unroll
    for (int w = 1; w < kLeakyWaves; ++w) t = MAX ? fmaxf(t, r[w]) : t + r[w];
    return t;
}

// y[row] = sum over the row's arcs of weight x x[column], every row of the direction (x, y and part in LDS; part: one
// float per piece of a long row).  Ends with the long rows' sums not yet formed: after a barrier, long_rows() does that.
__device__ __forceinline__ void sparse_product(const LeakyDir &d, const float *x, float *y, float *part)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (int i = wave; i < d.n_piece; i += kLeakyWaves) {
        const int e0 = d.piece_ptr[i] + lane, e1 = d.piece_ptr[i + 1];
        float w[kLeakyPiece / 64];
        int32_t c[kLeakyPiece / 64];
#pragma unroll
        for (int u = 0; u < kLeakyPiece / 64; ++u) {   // every load first
            const bool in = e0 + u * 64 < e1;
            w[u] = in ? d.long_w[e0 + u * 64] : 0.0f;
            c[u] = in ? d.long_src[e0 + u * 64] : 0;
        }
        float acc = 0.0f;
#pragma unroll
        for (int u = 0; u < kLeakyPiece / 64; ++u) acc = fmaf(w[u], x[c[u]], acc);
        acc = wsum(acc);
        if (lane == 0) part[i] = acc;
    }
    for (int j = 0; j < d.n_block; ++j) {
        const int r = d.short_row[(size_t)j * kLeakyThreads + tid];
        const int slots = d.block_slots[j];
        const int32_t *es = d.ell_src + d.block_off[j] + tid;
        const float *ew = d.ell_w + d.block_off[j] + tid;
        // four slots at a time, the next four on their way while these are added: eight loads in flight per thread
        float acc = 0.0f, w0[4], w1[4];
        int32_t c0[4], c1[4];
        if (slots > 0) {
#pragma unroll
            for (int u = 0; u < 4; ++u) { w0[u] = ew[(size_t)u * kLeakyThreads]; c0[u] = es[(size_t)u * kLeakyThreads]; }
        }
        for (int s = 0; s < slots; s += 4) {
            if (s + 4 < slots) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    w1[u] = ew[(size_t)(s + 4 + u) * kLeakyThreads];
                    c1[u] = es[(size_t)(s + 4 + u) * kLeakyThreads];
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) acc = fmaf(w0[u], x[c0[u]], acc);
#pragma unroll
            for (int u = 0; u < 4; ++u) { w0[u] = w1[u]; c0[u] = c1[u]; }
        }
        if (r >= 0) y[r] = acc;
    }
}
// the sums of the long rows from their pieces, in order (after a barrier behind sparse_product; before one)
__device__ __forceinline__ void long_rows(const LeakyDir &d, float *y, const float *part)
{
    for (int i = threadIdx.x; i < d.n_long; i += kLeakyThreads) {
        float acc = 0.0f;
        for (int p = d.long_piece[i]; p < d.long_piece[i + 1]; ++p) acc += part[p];
        y[d.long_row[i]] = acc;
    }
}

// What a thread needs of "its" states k = tid, tid + 1024, ... is the same in every frame and stays in registers.
constexpr int kLeakyPerThread = 8;    // states per thread: K <= 8192 (four float vectors of 10 000 states would not fit LDS anyway)

__global__ __launch_bounds__(kLeakyThreads) void fb_leaky_kernel(const LeakyParams P)
{
    extern __shared__ float lds[];
    const int tid = threadIdx.x, b = blockIdx.x;
    const int K = P.K, D = P.D, NT = kLeakyThreads;
    constexpr int U = kLeakyPerThread;
    const int Kp = (K + 3) & ~3, Dp = (D + 3) & ~3;
    float *x = lds, *y = x + Kp, *z = y + Kp, *pi = z + Kp, *er = pi + Kp, *red = er + Dp, *part = red + 2 * kLeakyWaves;
    const LeakyDev &G = P.G;
    const int T = min(max(P.lengths[b], 0), P.N);
    const float leak = P.leak;
    const float *em = P.emis + (size_t)b * P.N * D;
    float *rows = P.rows + (size_t)b * P.N * K;
    float *post = P.pdf_post + (size_t)b * P.N * D;
    int turn = 0;

    for (int n = T; n < P.N; ++n)
        for (int d = tid; d < D; d += NT) post[(size_t)n * D + d] = 0.0f;
    auto nothing = [&]() {   // a sequence without any path: log Z = -inf, no posteriors
        for (int n = 0; n < T; ++n)
            for (int d = tid; d < D; d += NT) post[(size_t)n * D + d] = 0.0f;
        if (tid == 0) P.logz[b] = -INFINITY;
    };
    if (T == 0) { nothing(); return; }

    uint32_t kpp[U];              // of state tid + u * 1024: its pdf | its place among the states in pdf order << 16
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const int k = tid + u * NT;
        const bool in = k < K;
        kpp[u] = in ? (uint32_t)G.pdf[k] | ((uint32_t)G.pos[k] << 16) : 0u;
        if (in) pi[k] = G.pi[k];   // (read back by this thread only)
    }

    // The emissions of a frame are asked for one step before they are needed (registers, up to kPre per thread).
    constexpr int kPre = 4;
    const bool pre = D <= kPre * NT;
    float pe[kPre];
    auto fetch = [&](int n) {
        if (pre) {
#pragma unroll
            for (int u = 0; u < kPre; ++u) pe[u] = tid + u * NT < D ? em[(size_t)n * D + tid + u * NT] : -INFINITY;
        }
    };
    // emissions of frame n (fetched before) -> er (in place after a barrier); next: the frame to fetch now, or -1
    auto stage = [&](int n, int next) {
        if (pre) {
#pragma unroll
            for (int u = 0; u < kPre; ++u)
                if (tid + u * NT < D) er[tid + u * NT] = pe[u];
            if (next >= 0) fetch(next);
        } else {
            for (int d = tid; d < D; d += NT) er[d] = em[(size_t)n * D + d];
        }
        __syncthreads();
    };
    // The scale of a frame's emission factors: the largest emission among the states that carry probability in vec (0
    // if there is none above zero-bar).  Not the largest of the row: a pdf that no state is tied to, or whose states are
    // out of reach in this frame, may lie far above the others, and factors relative to it would leave a float's range.
    auto frame_scale = [&](const float *vec) {
        float m = -INFINITY;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (tid + u * NT < K && vec[tid + u * NT] > 0.0f) m = fmaxf(m, er[kpp[u] & 0xffffu]);
        m = block_reduce<true>(m, red, turn);
        if (!(m > -INFINITY)) m = 0.0f;
        return m;
    };

    // ---- forward
    double log_scale = 0.0;
    float zl = 0.0f;
    fetch(0);
    for (int n = 0; n < T; ++n) {
        stage(n, n + 1 < T ? n + 1 : -1);
        if (n > 0) {
            sparse_product(G.fwd, x, y, part);   // x = previous vector with the leak handed out
            __syncthreads();
            long_rows(G.fwd, y, part);
        } else {
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (tid + u * NT < K) y[tid + u * NT] = G.initp[tid + u * NT];
        }
        __syncthreads();
        const float m = frame_scale(y);
        float s = 0.0f, v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = tid + u * NT;
            v[u] = 0.0f;
            if (k < K) {
                v[u] = y[k] * __expf(er[kpp[u] & 0xffffu] - m);
                s += v[u];
            }
        }
        s = block_reduce<false>(s, red, turn);
        if (!(s > 0.0f) || !(s < INFINITY)) { nothing(); return; }   // the same for every thread
        const float inv = 1.0f / s;
        float last = 0.0f;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int k = tid + u * NT;
            if (k < K) {
                const float a = v[u] * inv;
                rows[(size_t)n * K + k] = a;
                x[k] = a + leak * pi[k];                // the vector's sum is 1
                if (n == T - 1) last += a * G.finalp[k];
            }
        }
        log_scale += (double)logf(s) + (double)m;
        if (n == T - 1) zl = block_reduce<false>(last, red, turn);
        __syncthreads();   // x complete, er free
    }
    if (!(zl > 0.0f)) { nothing(); return; }
    if (tid == 0) P.logz[b] = log_scale + (double)logf(zl);

    // ---- backward: x = beta_n up to a factor; the forward vector of a frame is asked for one step before it is needed
    float pr[U];
    auto fetch_row = [&](int n) {
#pragma unroll
        for (int u = 0; u < U; ++u) pr[u] = tid + u * NT < K ? rows[(size_t)n * K + tid + u * NT] : 0.0f;
    };
    uint32_t drange[kPre];   // the states of pdf tid + j * 1024 in pdf order: begin | end << 16 (K < 65536)
#pragma unroll
    for (int j = 0; j < kPre; ++j) {
        const int d = tid + j * NT;
        drange[j] = d < D ? (uint32_t)G.pdf_ptr[d] | ((uint32_t)G.pdf_ptr[d + 1] << 16) : 0u;
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
        if (tid + u * NT < K) x[tid + u * NT] = G.finalp[tid + u * NT];
    fetch_row(T - 1);
    if (T >= 2) fetch(T - 1);
    __syncthreads();
    for (int n = T - 1; n >= 0; --n) {
        if (n < T - 1) {
            stage(n + 1, n >= 1 ? n : -1);
            const float m = frame_scale(x);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (tid + u * NT < K) y[tid + u * NT] = x[tid + u * NT] * __expf(er[kpp[u] & 0xffffu] - m);
            __syncthreads();
            sparse_product(G.bwd, y, z, part);
            __syncthreads();
            long_rows(G.bwd, z, part);
            __syncthreads();
            float c = 0.0f, tot = 0.0f, zv[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                zv[u] = tid + u * NT < K ? z[tid + u * NT] : 0.0f;
                if (tid + u * NT < K) c = fmaf(pi[tid + u * NT], zv[u], c);
                tot += zv[u];
            }
            c = block_reduce<false>(c, red, turn);
            tot = block_reduce<false>(tot, red, turn);
            const float add = leak * c, all = tot + (float)K * add;
            const float inv = all > 0.0f ? 1.0f / all : 0.0f;
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (tid + u * NT < K) x[tid + u * NT] = (zv[u] + add) * inv;
        }
        // the frame's posteriors, up to their sum, in pdf order: a pdf's states are neighbours
        float zn = 0.0f;
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (tid + u * NT < K) {
                const float p = pr[u] * x[tid + u * NT];   // (x[k]: written by this thread)
                y[kpp[u] >> 16] = p;
                zn += p;
            }
        if (n > 0) fetch_row(n - 1);
        zn = block_reduce<false>(zn, red, turn);   // (its barrier also puts y in place)
        const float inv = zn > 0.0f ? 1.0f / zn : 0.0f;
        if (pre) {
#pragma unroll
            for (int j = 0; j < kPre; ++j) {
                const int d = tid + j * NT;
                if (d < D) {
                    float acc = 0.0f;
                    for (int i = (int)(drange[j] & 0xffffu); i < (int)(drange[j] >> 16); ++i) acc += y[i];   // ascending states
                    post[(size_t)n * D + d] = acc * inv;
                }
            }
        } else {
            for (int d = tid; d < D; d += NT) {
                float acc = 0.0f;
                for (int i = G.pdf_ptr[d]; i < G.pdf_ptr[d + 1]; ++i) acc += y[i];
                post[(size_t)n * D + d] = acc * inv;
            }
        }
        __syncthreads();   // y and er free
    }
}

}  // namespace

size_t leaky_lds_bytes(int32_t K, int32_t D, int32_t n_piece)
{
    return ((size_t)((K + 3) & ~3) * 4 + (size_t)((D + 3) & ~3) + 2 * kLeakyWaves + (size_t)n_piece) * sizeof(float);
}

// Called once per shared graph with device copies (fb_graph_create): the row lists of both directions, pi, the
// initial and final weights as probabilities, the pdf tables.
int leaky_prepare(fb_graph *g, const float *init, const float *final_)
{
    const int32_t K = g->K;
    const HostLayout &L = g->lay;
    LeakyDev *dev = new LeakyDev();
    g->leaky = dev;
    int rc;
    if ((rc = build_dir(g, K, L.in_ptr, L.in_src, L.in_w, dev->fwd))) return rc;
    if ((rc = build_dir(g, K, L.out_ptr, L.out_dst, L.out_w, dev->bwd))) return rc;
    std::vector<float> pi((size_t)K), ip((size_t)K), fp((size_t)K);
    double top = -INFINITY, sum = 0.0;
    for (int32_t k = 0; k < K; ++k) top = std::max(top, (double)init[k]);
    for (int32_t k = 0; k < K; ++k) sum += top > -INFINITY ? std::exp((double)init[k] - top) : 0.0;
    for (int32_t k = 0; k < K; ++k) {
        pi[k] = sum > 0.0 ? (float)(std::exp((double)init[k] - top) / sum) : 0.0f;
        ip[k] = std::exp(init[k]);
        fp[k] = std::exp(final_[k]);
    }
    std::vector<int32_t> pdf((size_t)K), pos((size_t)K);
    for (int32_t d = 0; d < g->D; ++d)
        for (int32_t i = L.pdf_ptr[d]; i < L.pdf_ptr[d + 1]; ++i) {
            pdf[(size_t)L.pdf_states[i]] = d;
            pos[(size_t)L.pdf_states[i]] = i;
        }
    if ((rc = up(g, pi, &dev->pi)) || (rc = up(g, ip, &dev->initp)) || (rc = up(g, fp, &dev->finalp)) ||
        (rc = up(g, pdf, &dev->pdf)) || (rc = up(g, L.pdf_ptr, &dev->pdf_ptr)) || (rc = up(g, pos, &dev->pos)))
        return rc;
    return FB_OK;
}

void leaky_release(fb_graph *g)
{
    delete (LeakyDev *)g->leaky;
    g->leaky = nullptr;
}

}  // namespace fb

extern "C" {

size_t fb_leaky_workspace_bytes(const fb_graph *g, int32_t B, int32_t N)
{
    if (!g || g->n_seq != 0 || B <= 0 || N <= 0) return 0;
    return (((size_t)B * (size_t)N * (size_t)g->K * sizeof(float)) + 255) & ~(size_t)255;
}

int fb_leaky_posteriors(const fb_graph *g, const float *emis, const int32_t *lengths, int32_t B, int32_t N, int32_t D,
                        float leak, double *logz, float *pdf_post, void *ws, size_t ws_bytes, fb_stream stream)
{
    using namespace fb;
    if (!g) return fail(FB_EINVAL, "fb_leaky_posteriors: graph is NULL");
    if (g->host_only) return fail(FB_EINVAL, "fb_leaky_posteriors: graph was created with FB_GRAPH_HOST_ONLY");
    if (g->n_seq != 0) return fail(FB_EINVAL, "fb_leaky_posteriors: shared graphs only");
    if (!emis || !lengths || !logz || !pdf_post) return fail(FB_EINVAL, "fb_leaky_posteriors: NULL array");
    if (B <= 0 || N <= 0 || D <= 0) return fail(FB_EINVAL, "fb_leaky_posteriors: B, N and D must be positive");
    if (D != g->D) return fail(FB_EINVAL, "fb_leaky_posteriors: D differs from the graph's D");
    if (!(leak >= 0.0f) || !(leak <= 1.0f)) return fail(FB_EINVAL, "fb_leaky_posteriors: leak must lie in [0, 1]");
    if (!ws || ws_bytes < fb_leaky_workspace_bytes(g, B, N)) return fail(FB_EINVAL, "fb_leaky_posteriors: workspace missing or too small");
    if (!g->leaky) return fail(FB_EUNSUPPORTED, "fb_leaky_posteriors: the graph has no row lists for this mode");
    const LeakyDev &dev = *(const LeakyDev *)g->leaky;
    const size_t lds_bytes = leaky_lds_bytes(g->K, D, std::max(dev.fwd.n_piece, dev.bwd.n_piece));
    if (lds_bytes > kLdsBytes || g->K > kLeakyPerThread * kLeakyThreads || g->K > 65535)
        return fail(FB_EUNSUPPORTED, "fb_leaky_posteriors: more than 8192 states, or four state vectors and an emission row exceed the on-chip memory");
    LeakyParams p{};
    p.G = dev;
    p.emis = emis; p.lengths = lengths;
    p.B = B; p.N = N; p.D = D; p.K = g->K;
    p.leak = leak;
    p.logz = logz; p.pdf_post = pdf_post; p.rows = (float *)ws;
    if (lds_bytes > 64 * 1024) {
        const hipError_t e = hipFuncSetAttribute((const void *)fb_leaky_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return fail(FB_EHIP, std::string("hipFuncSetAttribute(LDS size): ") + hipGetErrorString(e));
    }
    hipLaunchKernelGGL(fb_leaky_kernel, dim3((unsigned)B), dim3(kLeakyThreads), lds_bytes, (hipStream_t)stream, p);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FB_EHIP, std::string("leaky-HMM kernel launch: ") + hipGetErrorString(e));
    return FB_OK;
}

}  // extern "C"
