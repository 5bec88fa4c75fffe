// gfx950 kernels of libfb_amd: the alpha / beta recursions (Eq. 13-14), the
// posteriors (Eq. 15) with their accumulation over tied states, and the LF-MMI
// objective (Eq. 16).
//
// Work decomposition.  Sequences of a batch are independent (the batched
// transition matrix is block diagonal), while the frames of one sequence are
// strictly sequential.  One workgroup therefore owns one (sequence, direction)
// pair for the whole time loop and keeps that sequence's state vector in LDS:
// a time step needs workgroup barriers only, never a grid-wide one, and the
// forward and backward recursions of a batch run side by side in one launch.
// Within a step the sparse product is walked one matrix row per lane along a
// static row-split sliced-ELL schedule (fb_sell.cpp) flattened into one stream of
// arcs per wave (fb_stream.cpp) that is prefetched several batches ahead; the arcs
// come from L2, the gathered vector from LDS.
//
// Arithmetic.  Internally logs are base 2 (weights and emissions are scaled by
// log2 e once), so the semiring sum is v_exp_f32 / v_log_f32 with no
// multiplications.  A row's (+)-sum is evaluated in one pass with a running
// maximum: one exponential per arc, one logarithm per row.  The state vector is
// kept normalised: every step subtracts the previous step's maximum, the
// subtracted amounts are the offsets handed back to the caller and their sum is
// accumulated in double for log Z.  The vector's element type ("carrier") is
// float or double; exponentials and logarithms are single precision either way
// (they act on differences to the running maximum, which are small).  One
// instantiation (LINW) takes the arc weights as 2^w and multiplies: see
// stream_linear_weights for when a graph gets it.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>
#include <utility>

#include "fb_internal.h"

namespace fb {

namespace {

constexpr float kNegBig = -1.0e30f;   // stands for "no finite term yet"; values below it count as semiring zero
constexpr double kLog2e = 1.4426950408889634074;
constexpr double kLn2 = 0.69314718055994530942;

__device__ __forceinline__ float fexp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float flog2(float x) { return __builtin_amdgcn_logf(x); }

// Maxima of values that are never NaN here: single instructions, without the quieting of
// signalling NaNs that fmaxf() implies.
__device__ __forceinline__ float tmax(float a, float b)
{
    float r;
    asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float tmin(float a, float b)
{
    float r;
    asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
    return r;
}
__device__ __forceinline__ float tmax3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
__device__ __forceinline__ double tmax(double a, double b) { return fmax(a, b); }
__device__ __forceinline__ double tmax3(double a, double b, double c) { return fmax(fmax(a, b), c); }

// running (+)-sum in base 2: value = m + log2(s); m in the carrier type, s single
template <class T>
__device__ __forceinline__ void lse_add(T &m, float &s, T x)
{
    const float d = (float)(x - m);
    const float e = fexp2(-fabsf(d));
    s = d > 0.0f ? fmaf(s, e, 1.0f) : s + e;
    m = tmax(m, x);
}

// four terms at once: one rescale of the running sum, then plain exponentials
template <class T>
__device__ __forceinline__ void lse_add4(T &m, float &s, T x0, T x1, T x2, T x3)
{
    const T mn = tmax3(tmax3(m, x0, x1), x2, x3);
    const float r = fexp2((float)(m - mn));
    const float e0 = fexp2((float)(x0 - mn)), e1 = fexp2((float)(x1 - mn));
    const float e2 = fexp2((float)(x2 - mn)), e3 = fexp2((float)(x3 - mn));
    s = fmaf(s, r, (e0 + e1) + (e2 + e3));
    m = mn;
}

// four terms whose weights are given as W = 2^w: the running maximum is over the gathered values alone
template <class T>
__device__ __forceinline__ void lse_add4w(T &m, float &s, T g0, T g1, T g2, T g3, float W0, float W1, float W2, float W3)
{
    const T mn = tmax3(tmax3(m, g0, g1), g2, g3);
    const float r = fexp2((float)(m - mn));
    float p = fexp2((float)(g0 - mn)) * W0;
    p = fmaf(fexp2((float)(g1 - mn)), W1, p);
    p = fmaf(fexp2((float)(g2 - mn)), W2, p);
    p = fmaf(fexp2((float)(g3 - mn)), W3, p);
    s = fmaf(s, r, p);
    m = mn;
}

template <class T>
__device__ __forceinline__ void lse_merge(T &m, float &s, T m2, float s2)
{
    const T M = tmax(m, m2);
    s = s * fexp2((float)(m - M)) + s2 * fexp2((float)(m2 - M));
    m = M;
}

// Data-parallel-primitive moves inside rows of 16 lanes, and reads of single lanes, for 32- and 64-bit values.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_u(uint32_t v)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) { return __uint_as_float(dpp_u<CTRL>(__float_as_uint(v))); }
template <int CTRL>
__device__ __forceinline__ double dpp_mov(double v)
{
    const uint64_t u = (uint64_t)__double_as_longlong(v);
    const uint64_t r = (uint64_t)dpp_u<CTRL>((uint32_t)u) | ((uint64_t)dpp_u<CTRL>((uint32_t)(u >> 32)) << 32);
    return __longlong_as_double((long long)r);
}
template <int CTRL>
__device__ __forceinline__ int dpp_mov(int v) { return (int)dpp_u<CTRL>((uint32_t)v); }
__device__ __forceinline__ int lane_value(int v, int l) { return __builtin_amdgcn_readlane(v, l); }
__device__ __forceinline__ float lane_value(float v, int l)
{
    return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(v), l));
}
__device__ __forceinline__ double lane_value(double v, int l)
{
    const uint64_t u = (uint64_t)__double_as_longlong(v);
    const uint64_t r = (uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)u, l) |
                       ((uint64_t)(uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(u >> 32), l) << 32);
    return __longlong_as_double((long long)r);
}

// v of every lane replaced by op over its aligned group of 2^lg lanes (lg = 1..6, the same in all
// lanes).  Inside a row of 16 lanes: exchanges with the lane whose number differs in one bit
// (the mirror moves equal that exchange once groups of 4 resp. 8 lanes hold one value); across
// rows: the four row results are read into scalars.
template <class V, class Op>
__device__ __forceinline__ V group_all(V v, int lg, int lane, Op op)
{
    v = op(v, dpp_mov<0xB1>(v));                  // quad_perm [1,0,3,2]
    if (lg >= 2) v = op(v, dpp_mov<0x4E>(v));     // quad_perm [2,3,0,1]
    if (lg >= 3) v = op(v, dpp_mov<0x141>(v));    // row_half_mirror
    if (lg >= 4) v = op(v, dpp_mov<0x140>(v));    // row_mirror
    if (lg >= 5) {
        const V lo = op(lane_value(v, 0), lane_value(v, 16)), hi = op(lane_value(v, 32), lane_value(v, 48));
        v = lg == 6 ? op(lo, hi) : (lane < 32 ? lo : hi);
    }
    return v;
}

// (m, s) of every lane replaced by the (+)-sum over its aligned group of 2^lg lanes (all lanes of
// the group end with the same pair): first the maximum, then the sums rescaled to it
template <class T>
__device__ __forceinline__ void group_total(T &m, float &s, int lg, int lane)
{
    const T mg = group_all(m, lg, lane, [](T a, T b) { return tmax(a, b); });
    s = group_all(s * fexp2((float)(m - mg)), lg, lane, [](float a, float b) { return a + b; });
    m = mg;
}

// Tropical semiring: the maximum over the group and the back-pointer of a lane that holds it
// (of the smallest back-pointer among those lanes, so the choice does not depend on timing).
template <class T>
__device__ __forceinline__ void group_best(T &m, int &arg, int lg, int lane)
{
    const T mg = group_all(m, lg, lane, [](T a, T b) { return tmax(a, b); });
    arg = group_all(m == mg ? arg : 0x7fffffff, lg, lane, [](int a, int b) { return min(a, b); });
    m = mg;
}

// reductions over the whole wave; every lane gets the result
template <class T>
__device__ __forceinline__ T wave_max(T v)
{
    return group_all(v, 6, (int)(threadIdx.x & (kWave - 1)), [](T a, T b) { return tmax(a, b); });
}

__device__ __forceinline__ float wave_sum(float v)
{
    return group_all(v, 6, (int)(threadIdx.x & (kWave - 1)), [](float a, float b) { return a + b; });
}

}  // namespace

// ---------------------------------------------------------------------------
// alpha / beta recursion.  grid = B * n_dir workgroups of NW waves; workgroup
// (b, which) runs direction dir[which] of sequence b over all its frames.
//
// With x_n the vector kept in LDS, both directions are the same recursion on a
// matrix and its transpose:
//   forward   x_n = alpha_n              = v_n o (+)_{in(j)}  (w (x) x_{n-1}[src])
//   backward  x_n = beta_n (x) v_n       = v_n o (+)_{out(i)} (w (x) x_{n+1}[dst])
// and beta_n itself is the row sum before v_n is applied.
//
// Waves 0..NW-2 compute: their only global-memory traffic inside the time loop
// is their own arc stream, a fixed sequence of loads that stays ahead of its
// use across barriers and across time steps; the LDS gathers of a batch are
// issued one batch ahead of the arithmetic that consumes them.  Wave NW-1 moves
// data: it brings the next frame's emissions from HBM straight into LDS, copies
// the finished vector of the previous step out, keeps the offsets and log Z.
// HBM latency therefore never sits in front of an arc load.
//
// LDS of a workgroup (carrier type T unless noted):
//   xb   2 x Xs   x of the previous / current step; Xs = Kcap + Ccap + 1: the
//                 states, then the clones of rows too long for one slice, then a dump slot
//   bh   2 x Xs   beta before v is applied (backward direction only)
//   red  4 x NW   step maxima, scratch of the last reduction.  Float vectors: the maximum of step i is
//                 word i % 3, reached by one LDS atomic maximum per wave; the data-moving wave clears
//                 the word of the step after next.  Double vectors: one slot per wave and parity.
//   er   3 x (Ecap + 1) float   emissions as given (natural log) of the frame in use and
//                               of the next two; slot Ecap = 0
//   pix  Ecap int32             packed graphs: pdf id of every state
//   vix  Xs uint16              which staged emission every target (state, clone, dump slot) takes
//   bpb  2 x Xs uint16          tropical semiring only: back-pointers of the previous / current step
//
// XF != 0: the state buffers have the fixed length XF (>= Kcap + Ccap + 1) whatever the graph.  The
// time loop is then unrolled over the two buffer parities, every buffer address is a compile-time
// constant, and a gather is one ds_read whose address register is the arc's source field as stored
// (a byte offset) with the buffer in the instruction's offset field.
// ---------------------------------------------------------------------------
// f(integral_constant<int, 0>), f(integral_constant<int, 1>), ...: a loop whose counter is a compile-time constant
template <class F, int... I>
__device__ __forceinline__ void unrolled(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}

// Workgroup -> (sequence, direction).  Workgroups start in the order of their index.  In the large-graph
// kernels (one workgroup fills a compute unit) the longest sequences therefore come first, both
// directions of a sequence side by side: whatever delays the start of a workgroup - a second wave of
// workgroups when there are more than compute units, workgroups of another launch in the way - then
// falls on the sequences that have time to spare.
// (A launch may cover only a range of ranks, P.order then holds the sequences in order of length.)
template <int NW>
__device__ __forceinline__ void resolve_sequence(const RecParams &P, double *lds_raw, int &b, int &which)
{
    constexpr int NT = NW * kWave;
    const int tid = threadIdx.x;
    const int n_launch = P.order ? P.n_launch : P.B;
    b = blockIdx.x % n_launch;
    which = blockIdx.x / n_launch;
    if (NW == kNWShared || P.order) {   // in order of length: both directions of a sequence side by side
        which = blockIdx.x % P.n_dir;
        b = blockIdx.x / P.n_dir;
    }
    if (P.order) {
        b = P.order[P.rank0 + b];
    } else if (NW == kNWShared) {
        const int r = b;   // this workgroup takes the sequence of rank r by length
        int *sel = (int *)lds_raw;
        for (int cand = tid; cand < P.B; cand += NT) {
            const int lc = min(max(P.lengths[cand], 0), P.N);
            int rank = 0;   // sequences that go before cand: the longer ones, and of the equally long the earlier ones
            for (int j = 0; j < P.B; ++j) {
                const int lj = min(max(P.lengths[j], 0), P.N);
                rank += (lj > lc || (lj == lc && j < cand)) ? 1 : 0;
            }
            if (rank == r) *sel = cand;
        }
        __syncthreads();
        b = __builtin_amdgcn_readfirstlane(*sel);
        __syncthreads();   // the word is part of a state buffer from here on
    }
}

// Progress counter of a launch: everything this workgroup writes is on its way; make it visible device-wide, then count.
__device__ __forceinline__ void count_done(const RecParams &P)
{
    if (P.done) {
        const int rank = P.rank0 + (int)blockIdx.x / P.n_dir;   // (launches with counters cover ranks in order)
        int slot = 0;
#pragma unroll
        for (int i = 0; i < kDoneCuts; ++i) slot += rank >= P.done_from[i] ? 1 : 0;
        __syncthreads();
        if (threadIdx.x == 0 && slot > 0) {
            __threadfence();
            atomicAdd(P.done + slot, 1u);
        }
    }
}

// One (sequence, direction) pair from its first frame to its last, by the whole workgroup.
template <int NW, class T, bool TROP, int XF, bool LINW = false>
__device__ __forceinline__ void recursion_run(const RecParams &P, const int b, const int which, double *lds_raw)
{
    static_assert(!LINW || (!TROP && XF != 0), "weights as 2^w: log semifield, fixed buffers");
    constexpr int NRES = kResident;
    constexpr int NT = NW * kWave, NC = NW - 1;
    const T kNegInf = (T)(-INFINITY);
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool io_wave = wave == NC;
    const RecDir &R = P.dir[which];
    const StreamDev &S = R.sched;
    const bool bwd = R.backward != 0;
    const SubDesc sd = S.sub[P.shared ? 0 : b];
    const int K = sd.K, k0 = sd.k0, nC = sd.n_slot;
    const int Tn = min(max(P.lengths[b], 0), P.N);
    const int nE = P.shared ? P.D : K;           // entries of a staged emission vector
    const int nX = P.Kcap + R.Ccap + 1;          // states, clone slots, dump slot
    const int Xs = XF ? XF : nX, Es = P.Ecap + 1;

    T *xb = (T *)lds_raw;
    T *bh = xb + 2 * Xs;
    T *red = bh + (bwd ? 2 * Xs : 0);
    float *er = (float *)(red + 4 * NW + 2);
    int32_t *pix = (int32_t *)(er + 3 * Es);
    uint16_t *vix = (uint16_t *)(pix + (P.shared ? 0 : P.Ecap));   // emission index of every target
    uint16_t *bpb = vix + ((Xs + 1) & ~1);                         // tropical semiring: 2 x Xs back-pointers
    constexpr int kSrcShift = sizeof(T) == 4 ? 2 : 3;              // an arc's source field is index << kSrcShift

    const float *em_seq = P.emis + (size_t)b * P.N * P.D;
    const size_t out_ld = P.shared ? (size_t)(R.out_ld ? R.out_ld : K) : (size_t)P.Ktot;
    const size_t out_at = P.shared ? (size_t)b * P.N * out_ld : (size_t)k0;
    float *out_f = (R.out && !R.out_carrier) ? (float *)R.out + out_at : nullptr;
    T *out_t = (R.out && R.out_carrier) ? (T *)R.out + out_at : nullptr;
    double *off_seq = R.off ? R.off + (size_t)b * P.N : nullptr;
    auto frame = [&](int i) { return bwd ? Tn - 1 - i : i; };
    // the maximum over the workgroup of the vector of step i (the next step normalises by it)
    constexpr bool kAtomMax = sizeof(T) == 4;
    auto put_max = [&](int i, T wmax) {
        // (a double carrier's maximum is reduced as a float rounded up: what the next step subtracts from every entry
        // need only be near the largest, the same for all, and not below it by more than rounding)
        if constexpr (sizeof(T) == 8) wmax = (T)wave_max(__double2float_ru((double)wmax));
        else wmax = wave_max(wmax);
        if (lane == 0) {   // (one lane per wave: atomics of many lanes on one word are served one at a time)
            if constexpr (kAtomMax)
                __builtin_amdgcn_ds_fmaxf((__attribute__((address_space(3))) float *)(red + i % 3), (float)wmax, 0, 0, false);
            else
                red[(i & 1) * NW + wave] = wmax;
        }
    };
    auto get_max = [&](int i) {
        if constexpr (kAtomMax) {
            return red[i % 3];
        } else {
            T M = red[(i & 1) * NW];
#pragma unroll
            for (int w = 1; w < NW; ++w) M = tmax(M, red[(i & 1) * NW + w]);
            return M;
        }
    };

    // ---- duties of the data-moving wave (called by that wave only, all 64 lanes)
    // Packed graphs: the pdf of the lane's states u * 64 + lane, in registers when a (sub-)graph has at most
    // kPixRegs * 64 states (read once: looked up in LDS at every frame, each of a frame's loads would wait for a read)
    // (the small-graph instantiations only: the others have no registers to spare)
    constexpr int kPixRegs = NW == kNWSmall ? 8 : 0;
    const bool pix_in_regs = kPixRegs > 0 && !P.shared && nE <= kPixRegs * kWave;
    int32_t pixr[kPixRegs > 0 ? kPixRegs : 1] = {};
    // emissions of frame f -> dst, through the direct global->LDS path (no registers, any length)
    auto stage = [&](int f, float *dst) {
        const float *row = em_seq + (size_t)f * P.D;
        if (P.shared) {
            if ((P.D & 3) == 0 && ((uintptr_t)row & 15) == 0) {
                for (int e0 = 0; e0 < nE; e0 += 4 * kWave)
                    if (e0 + 4 * lane < nE)
                        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(row + e0 + 4 * lane),
                                                         (__attribute__((address_space(3))) void *)(dst + e0), 16, 0, 0);
            } else {
                for (int e0 = 0; e0 < nE; e0 += kWave)
                    if (e0 + lane < nE)
                        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(row + e0 + lane),
                                                         (__attribute__((address_space(3))) void *)(dst + e0), 4, 0, 0);
            }
        } else if (kPixRegs > 0 && pix_in_regs) {
#pragma unroll
            for (int u = 0; u < kPixRegs; ++u)
                if (u * kWave < nE && u * kWave + lane < nE)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(row + pixr[u]),
                                                     (__attribute__((address_space(3))) void *)(dst + u * kWave), 4, 0, 0);
        } else {
            for (int e0 = 0; e0 < nE; e0 += kWave)
                if (e0 + lane < nE)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(row + pix[e0 + lane]),
                                                     (__attribute__((address_space(3))) void *)(dst + e0), 4, 0, 0);
        }
    };
    auto staged_wait = [&]() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };
    // a finished vector -> global memory, coalesced; a cloned state leaves as the (+)-sum of its clones
    const CloneDesc *cdesc = S.clones + sd.clone0;
    // (copies go in groups of several pieces per lane, all read before any is stored: a store's data registers
    // can only be reused once the store has completed, so a read-one-store-one loop would pay a full HBM
    // round trip per piece)
    auto copy_out = [&](auto *orow, const auto *srcv, int n, auto cvt) {
        constexpr int U = NW == kNWShared ? 16 : 8;   // (small graphs: a row of up to 512 states is one group)
        for (int k0 = 0; k0 < n; k0 += U * kWave) {
            std::remove_cv_t<std::remove_reference_t<decltype(srcv[0])>> v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = srcv[min(k0 + u * kWave + lane, n - 1)];
#pragma unroll
            for (int u = 0; u < U; ++u) asm volatile("" : "+v"(v[u]));   // every read stays in front of the stores
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (k0 + u * kWave + lane < n) orow[k0 + u * kWave + lane] = cvt(v[u]);
        }
    };
    auto write_row = [&](int f, const T *srcv) {
        if (out_f) {
            float *orow = out_f + (size_t)f * out_ld;
            const float scale = R.out_scale;
            copy_out(orow, srcv, K, [scale](T x) { return (float)x * scale; });
        } else if (out_t) {
            T *orow = out_t + (size_t)f * out_ld;
            if (sizeof(T) == 4 && (out_ld & 3) == 0 && (size_t)((K + 3) & ~3) <= out_ld && ((uintptr_t)orow & 15) == 0 &&
                ((uintptr_t)srcv & 15) == 0) {
                // whole 16-byte pieces; when K is not a multiple of 4 the last one takes up to 3 values that lie
                // behind the states in LDS into the row's padding, which nobody reads
                const float4 *s4 = (const float4 *)srcv;
                float4 *o4 = (float4 *)orow;
                constexpr int U = 8;
                const int n4 = (K + 3) / 4;
                for (int k0 = 0; k0 < n4; k0 += U * kWave) {
                    float4 v[U];
#pragma unroll
                    for (int u = 0; u < U; ++u) v[u] = s4[min(k0 + u * kWave + lane, n4 - 1)];
#pragma unroll
                    for (int u = 0; u < U; ++u)   // every read stays in front of the stores
                        asm volatile("" : "+v"(v[u].x), "+v"(v[u].y), "+v"(v[u].z), "+v"(v[u].w));
#pragma unroll
                    for (int u = 0; u < U; ++u)
                        if (k0 + u * kWave + lane < n4) o4[k0 + u * kWave + lane] = v[u];
                }
            } else {
                copy_out(orow, srcv, K, [](T x) { return x; });
            }
        }
        if (out_f || out_t)
            for (int j = lane; j < sd.n_cdesc; j += kWave) {   // stores of one wave to one address keep their order
                const CloneDesc cd = cdesc[j];
                T m = (T)kNegBig;
                float s = 0.0f;
                lse_add(m, s, srcv[cd.state]);
                for (int i = 0; i < cd.count; ++i) lse_add(m, s, srcv[P.Kcap + cd.first + i]);
                const T v = m + (T)flog2(s);
                if (out_f) out_f[(size_t)f * out_ld + cd.state] = (float)v * R.out_scale;
                else out_t[(size_t)f * out_ld + cd.state] = v;
            }
    };

    // tropical semiring: the back-pointers of frame f (f >= 1) -> global memory; a row holds the states
    // and, behind them, the clone slots (a back-pointer is an index into the state buffer: a state, or
    // Kcap + slot for a clone)
    auto write_bp = [&](int f, const uint16_t *srcb) {
        if (TROP && R.bp) {
            uint16_t *orow = R.bp + (P.shared ? ((size_t)b * P.N + f) * R.bp_ld : (size_t)f * R.bp_ld);
            uint16_t *ost = orow + (P.shared ? 0 : k0), *ocl = orow + (P.shared ? K : P.Ktot + b * R.Ccap);
            copy_out(ost, srcb, K, [](uint16_t x) { return x; });
            copy_out(ocl, srcb + P.Kcap, nC, [](uint16_t x) { return x; });
        }
    };

    if (Tn > 0) {
        // ---- first frame of this direction: x = start weight (x) v
        if (!P.shared)
            for (int k = tid; k < K; k += NT) pix[k] = P.pdf[k0 + k];
        for (int k = tid; k < nX; k += NT) vix[k] = S.vix[(size_t)(P.shared ? 0 : b) * nX + k];
        if (tid < 3) er[tid * Es + P.Ecap] = 0.0f;   // the emission of rows that take none
        if (kAtomMax && tid < 3) red[tid] = kNegInf;
        __syncthreads();
        if (io_wave) {
            if (kPixRegs > 0 && pix_in_regs) {
#pragma unroll
                for (int u = 0; u < kPixRegs; ++u) pixr[u] = u * kWave + lane < nE ? pix[u * kWave + lane] : 0;
            }
            stage(frame(0), er);
            if (Tn > 1) stage(frame(1), er + Es);
            staged_wait();
            if (Tn > 2) stage(frame(2), er + 2 * Es);   // lands while step 1 runs
            if (off_seq && lane == 0) off_seq[frame(0)] = 0.0;
            if (R.cum && lane == 0) R.cum[(size_t)b * P.N + frame(0)] = 0.0f;
        }
        __syncthreads();
        T wmax = kNegInf;
        for (int k = tid; k < K; k += NT) {
            const T s = (T)R.bound[k0 + k];
            const T x = s + (T)er[P.shared ? P.pdf[k0 + k] : k] * (T)kLog2e;
            xb[k] = x;
            if (bwd) bh[k] = s;
            wmax = tmax(wmax, x);
        }
        for (int k = tid; k < nC; k += NT) {   // clones start empty: the state itself holds the start weight
            xb[P.Kcap + k] = kNegInf;
            if (bwd) bh[P.Kcap + k] = kNegInf;
        }
        if (tid == 0) xb[nX - 1] = xb[Xs + nX - 1] = kNegInf;   // the dump slot holds zero-bar in both buffers, always
        put_max(0, wmax);
        __syncthreads();

        double csum = 0.0;
        if (io_wave) {
            for (int i = 1; i < Tn; ++i) {
                const int cur = (i - 1) & 1;
                const T M = get_max(i - 1);
                const T c = (M == kNegInf) ? (T)0 : M;
                csum += (double)c;
                if (off_seq && lane == 0) off_seq[frame(i)] = csum * (double)R.out_scale;
                if (R.cum && lane == 0) R.cum[(size_t)b * P.N + frame(i)] = (float)csum;
                staged_wait();   // frame i+1, requested a whole step ago, is in LDS
                if (i + 2 < Tn) stage(frame(i + 2), er + ((i + 2) % 3) * Es);   // buffer of frame i-1: no longer read
                write_row(frame(i - 1), bwd ? bh + cur * Xs : xb + cur * Xs);
                if (TROP && i >= 2) write_bp(i - 1, bpb + cur * Xs);
                if (lane == 0) {   // its own slot counts for nothing / the word of step i + 1 starts empty
                    if (kAtomMax) red[(i + 1) % 3] = kNegInf;
                    else red[(i & 1) * NW + wave] = kNegInf;
                }
                __syncthreads();
            }
        } else {
            const WaveDesc wd = S.waves[sd.wave_ptr0 + wave];
            // a lane's share of a batch is two 16-byte pieces: rows 0-1 and rows 2-3
            // (the address is a wave-uniform base plus the lane's 16 bytes: no per-lane 64-bit arithmetic)
            const uint64_t arc_base = (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)wd.arc_base) |
                                      ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(wd.arc_base >> 32)) << 32);
            const float4 *stream = (const float4 *)(S.arcs + arc_base);
            auto load_from = [&](Arc(&dst)[kBatchRows], const float4 *p) {   // p: the lane's first piece
                const float4 lo = p[0], hi = p[kWave];
                dst[0] = Arc{(int32_t)__float_as_uint(lo.x), lo.y};
                dst[1] = Arc{(int32_t)__float_as_uint(lo.z), lo.w};
                dst[2] = Arc{(int32_t)__float_as_uint(hi.x), hi.y};
                dst[3] = Arc{(int32_t)__float_as_uint(hi.z), hi.w};
            };
            // The first NRES batches of the wave's step stay in registers for the whole time loop;
            // the rest of the stream is re-read every step through a ring that runs kRing-1 batches
            // ahead of its use, across barriers and across steps (it holds graph data only).
            Arc res[NRES][kBatchRows];
#pragma unroll
            for (int q = 0; q < NRES; ++q) load_from(res[q], stream + (size_t)q * (2 * kWave) + lane);
            // streamed part: rp0 = the lane's piece of its first batch, rp = of the batch to request next (the
            // requests walk the part cyclically, so the pointer moves by one batch per request and goes back
            // to rp0 once per time step, at a place every step knows: no index arithmetic per batch)
            const float4 *const rp0 = stream + (size_t)NRES * (2 * kWave) + lane;
            const float4 *rp = rp0;
            const int n_iter = wd.n_iter;
            // flag bytes: words 0-1 of the wave hold those of the resident batches, then one word per
            // iteration; kept in registers (word i in lane i) and read with v_readlane
            const uint32_t *fwp = S.flagwords + wd.flag_base;
            const uint32_t rflag0 = fwp[0], rflag1 = fwp[1];
            // batches of the resident part that hold arcs (padding only follows them, and only when nothing is streamed)
            int n_res = 0;
            for (int q = 0; q < NRES; ++q)
                if (!((((q < 4 ? rflag0 : rflag1) >> (8 * (q & 3))) & 0xffu) & kFlagSkip)) n_res = q + 1;
            n_res = __builtin_amdgcn_readfirstlane(n_res);
            const uint32_t fwv0 = lane < n_iter ? fwp[2 + lane] : 0u;
            const uint32_t fwv1 = lane + kWave < n_iter ? fwp[2 + lane + kWave] : 0u;
            Arc ring[kRing][kBatchRows];
            if (n_iter > 0) {
#pragma unroll
                for (int j = 0; j + 1 < kRing; ++j) {
                    load_from(ring[j], rp);
                    rp += 2 * kWave;
                    __builtin_amdgcn_sched_barrier(0);   // keep the issue order: waits count loads in order
                }
            }
            // gathered values of the batch being folded and of the next one; the buffers rotate with the batch
            // number, and an unrolled iteration must bring the rotation back to where it started
            constexpr int GB = kRing % 2 == 0 ? 2 : 3;
            static_assert(kRing % GB == 0, "ring size must be a multiple of the gather buffer count");
            T g[GB][kBatchRows];
            // Source fields are byte offsets into the buffer vbase.  With fixed buffers the workgroup's LDS
            // starts at address 0 (the host launches this instantiation only if the kernel has no static LDS)
            // and the buffer sits at a constant address, so the load takes the field itself as its address.
            // The source field of a batch's last row carries the row's target in its upper half when the batch
            // closes a slice (zero otherwise: offsets stay below 64 KB), so its lower half is the source either way.
            // stacked: the batch holds the rows of several stacked slices, whose parts all end with a target in
            // the upper half (only the first kMaxStacked batches of a step can be: the flag is a constant false elsewhere)
            auto gather = [&](T(&dst)[kBatchRows], const Arc(&a)[kBatchRows], const T *vbase, bool stacked) {
                auto at = [&](int32_t off) {
                    if constexpr (XF != 0) {
                        typedef const __attribute__((address_space(3))) T lds_ct;
                        const uint32_t addr = (uint32_t)off + (vbase == xb ? 0u : (uint32_t)(XF * sizeof(T)));
                        return *(lds_ct *)(uintptr_t)addr;
                    } else {
                        return *(const T *)((const char *)vbase + off);
                    }
                };
                if (stacked) {
#pragma unroll
                    for (int r = 0; r < kBatchRows; ++r) {
                        uint32_t s = (uint32_t)a[r].src;
                        asm volatile("" : "+v"(s));   // (not hoisted out of the time loop: see target() below)
                        dst[r] = at((int32_t)(s & 0xffffu));
                    }
                } else {
#pragma unroll
                    for (int r = 0; r + 1 < kBatchRows; ++r) dst[r] = at(a[r].src);
                    dst[kBatchRows - 1] = at((int32_t)((uint32_t)a[kBatchRows - 1].src & 0xffffu));
                }
            };

            // one time step; curc: parity of the buffer that holds the previous step (an int, or a
            // compile-time constant when the buffers have fixed addresses)
            auto step = [&](int i, auto curc) {
                const int cur = curc, nxt = cur ^ 1;
                const T *xc = xb + cur * Xs;
                T *xn = xb + nxt * Xs;
                T *bn = bh + nxt * Xs;
                const float *ern = er + (i % 3) * Es;
                // Waves of equal priority are served oldest first, so with one fixed priority the younger waves of
                // a SIMD would do most of their step alone after the older ones have finished theirs.  A wave's
                // priority therefore falls as its step advances: whoever has more left goes first, and the waves
                // of a SIMD reach the barrier together.  The younger half of the waves stays one level above the
                // older half, which would otherwise still win every tie.
                const bool young = wave >= NW / 2;
                auto prio = [&](auto level) {   // level: a compile-time constant 1..3
                    if (NW == kNWShared) {
                        if (young) __builtin_amdgcn_s_setprio(decltype(level)::value);
                        else __builtin_amdgcn_s_setprio(decltype(level)::value - 1);
                    }
                };
                prio(std::integral_constant<int, 3>{});
                const T M = get_max(i - 1);
                const T c = (M == kNegInf) ? (T)0 : M;
                wmax = kNegInf;
                T m = TROP ? kNegInf : (T)kNegBig;
                float sum = 0.0f;
                int arg = 0;                         // tropical semiring: the state the best term so far came from
                uint16_t *bpn = bpb + nxt * Xs;
                const T *vbase = xc;
                if (i <= 2)   // rows without arcs: the semiring zero from the second frame on, in both buffers
                    for (int z = tid; z < sd.n_zero; z += NC * kWave) {
                        const int k = S.zero_rows[sd.zero0 + z];
                        xn[k] = kNegInf;
                        if (bwd) bn[k] = kNegInf;
                    }
                // fold one batch: a, gv = its entries and gathered values; next = the batch after it (its
                // gathers are issued before this batch's arithmetic), has_next: there is one
                // res: the batch is one of the first kMaxStacked of the step (the only ones that may be stacked);
                // next_stacked: the batch after it is a stacked one
                auto fold = [&](auto res, uint32_t f, const Arc(&a)[kBatchRows], const T(&gv)[kBatchRows], T(&gnext)[kBatchRows],
                                const Arc(&next)[kBatchRows], bool next_stacked, bool has_next) {
                    if (has_next) gather(gnext, next, vbase, next_stacked);
                    if (decltype(res)::value && (f & (kFlagDual | kFlagQuad))) {
                        // Stacked slices: every part of the lane is a row of its own with one or two terms, closed
                        // here; the running sums of the lane are not touched (stacked batches come first).
                        // val: the part's (+)-sum; parg: tropical semiring, where its best term came from
                        // The emissions of the parts' targets first, all of them (two LDS reads in a row each, one
                        // after the other per part they would be most of a small graph's time step).
                        const bool quad = (f & kFlagQuad) != 0;
                        uint32_t ptgt[kBatchRows];
                        float pem[kBatchRows];
#pragma unroll
                        for (int r = 0; r < kBatchRows; ++r) {
                            uint32_t field = (uint32_t)a[(quad || (r & 1)) ? r : r + 1].src;   // two parts: rows 1 and 3 name the targets
                            asm volatile("" : "+v"(field));
                            ptgt[r] = field >> 16;
                        }
                        uint32_t pvi[kBatchRows];
#pragma unroll
                        for (int r = 0; r < kBatchRows; ++r) pvi[r] = vix[ptgt[r]];
#pragma unroll
                        for (int r = 0; r < kBatchRows; ++r) pem[r] = ern[pvi[r]];
                        auto close_part = [&](T val, int parg, int r) {   // r: a row of the part that names its target
                            const uint32_t tgt = ptgt[r];
                            const T pre = val - c;
                            const T x = pre + (T)pem[r] * (T)kLog2e;
                            xn[tgt] = x;
                            if constexpr (TROP) bpn[tgt] = (uint16_t)(parg >> kSrcShift);
                            else if (bwd) bn[tgt] = pre;
                            wmax = tmax(wmax, x);
                        };
                        T xs[kBatchRows];
#pragma unroll
                        for (int r = 0; r < kBatchRows; ++r) xs[r] = gv[r] + (T)a[r].w;
                        if (f & kFlagQuad) {
#pragma unroll
                            for (int r = 0; r < kBatchRows; ++r) {   // one term: the sum is the term
                                const uint32_t field = (uint32_t)a[r].src;
                                if constexpr (TROP) close_part(xs[r], xs[r] > kNegInf ? (int)(field & 0xffffu) : 0, r);
                                else close_part(xs[r] > (T)kNegBig ? xs[r] : kNegInf, 0, r);   // (as the running sums treat it)
                            }
                        } else {
#pragma unroll
                            for (int p = 0; p < 2; ++p) {
                                const T u0 = xs[2 * p], u1 = xs[2 * p + 1];
                                const uint32_t field = (uint32_t)a[2 * p + 1].src;
                                if constexpr (TROP) {
                                    T pm = kNegInf;
                                    int parg = 0;
                                    if (u0 > pm) { pm = u0; parg = a[2 * p].src; }
                                    if (u1 > pm) { pm = u1; parg = (int)(field & 0xffffu); }
                                    close_part(pm, parg, 2 * p + 1);
                                } else {
                                    const T pm = tmax3((T)kNegBig, u0, u1);
                                    close_part(pm + (T)flog2(fexp2((float)(u0 - pm)) + fexp2((float)(u1 - pm))), 0, 2 * p + 1);   // 0 -> -inf
                                }
                            }
                        }
                    } else if (!(f & kFlagSkip)) {
                        const bool closing = (f & kFlagInfo) != 0;
                        const uint32_t last = (uint32_t)a[3].src;   // closing: source | target << 16
                        // the target, opaque to the optimiser: for the batches that stay in registers it would
                        // otherwise keep every target's addresses in registers of their own across the time loop
                        auto target = [&]() {
                            uint32_t v = last;
                            asm volatile("" : "+v"(v));
                            return v >> 16;
                        };
                        if constexpr (LINW) {
                            // weights as 2^w: a multiply-add per term in place of the add before the exponential;
                            // arcs of weight zero-bar gather the dump slot (zero-bar) and never raise the maximum
                            lse_add4w(m, sum, gv[0], gv[1], gv[2], gv[3], a[0].w, a[1].w, a[2].w, a[3].w);
                            if (closing) {
                                const int lg = (int)((f >> kFlagLgShift) & 7u);
                                if (lg) group_total(m, sum, lg, lane);
                                const uint32_t tgt = target();
                                const T pre = m + (T)flog2(sum) - c;   // sum == 0 -> -inf
                                const T x = pre + (T)ern[vix[tgt]] * (T)kLog2e;
                                xn[tgt] = x;
                                if (bwd) bn[tgt] = pre;
                                wmax = tmax(wmax, x);
                                m = (T)kNegBig;
                                sum = 0.0f;
                            }
                            return;
                        }
                        const T x0 = gv[0] + (T)a[0].w, x1 = gv[1] + (T)a[1].w, x2 = gv[2] + (T)a[2].w, x3 = gv[3] + (T)a[3].w;
                        if constexpr (TROP) {
                            // (+) = max: keep the largest term and the state it came from (the first of equal terms)
                            auto take = [&](T x, int s) {
                                if (x > m) { m = x; arg = s; }
                            };
                            take(x0, a[0].src);
                            take(x1, a[1].src);
                            take(x2, a[2].src);
                            take(x3, (int)(last & 0xffffu));
                            if (closing) {
                                const int lg = (int)((f >> kFlagLgShift) & 7u);
                                if (lg) group_best(m, arg, lg, lane);
                                const uint32_t tgt = target();
                                const T x = (m - c) + (T)ern[vix[tgt]] * (T)kLog2e;
                                xn[tgt] = x;
                                bpn[tgt] = (uint16_t)(arg >> kSrcShift);
                                wmax = tmax(wmax, x);
                                m = kNegInf;
                                arg = 0;
                            }
                        } else {
                            lse_add4(m, sum, x0, x1, x2, x3);
                            if (closing) {   // the rows' sums are complete
                                const int lg = (int)((f >> kFlagLgShift) & 7u);
                                if (lg) group_total(m, sum, lg, lane);   // the row's arcs were spread over 2^lg lanes
                                const uint32_t tgt = target();
                                const T pre = m + (T)flog2(sum) - c;   // sum == 0 -> -inf
                                const T x = pre + (T)ern[vix[tgt]] * (T)kLog2e;
                                xn[tgt] = x;
                                if (bwd) bn[tgt] = pre;
                                wmax = tmax(wmax, x);
                                m = (T)kNegBig;
                                sum = 0.0f;
                            }
                        }
                    }
                };
                auto rflag = [&](int q) { return ((q < 4 ? rflag0 : rflag1) >> (8 * (q & 3))) & 0xffu; };
                const uint32_t fw_first = n_iter > 0 ? (uint32_t)__builtin_amdgcn_readlane(fwv0, 0) : 0u;
                auto is_stacked = [&](uint32_t f) { return (f & (kFlagDual | kFlagQuad)) != 0; };
                gather(g[0], res[0], vbase, is_stacked(rflag(0)));
                unrolled([&](auto qc) {
                    constexpr int q = decltype(qc)::value;
                    if (q < n_res) {   // (a small graph fills only the first of them: the padding behind is not walked)
                        if constexpr (q + 1 < NRES)
                            fold(std::bool_constant<(q < kMaxStacked)>{}, rflag(q), res[q], g[q % GB], g[(q + 1) % GB], res[q + 1],
                                 q + 1 < kMaxStacked && is_stacked(rflag(q + 1)), q + 1 < n_res);
                        else
                            fold(std::bool_constant<(q < kMaxStacked)>{}, rflag(q), res[q], g[q % GB], g[(q + 1) % GB], ring[0], false, n_iter > 0);
                    }
                }, std::make_integer_sequence<int, NRES>{});
                uint32_t fw = fw_first;
                prio(std::integral_constant<int, 2>{});
                for (int it = 0; it < n_iter; ++it) {
                    if (it == (n_iter + 1) / 2) prio(std::integral_constant<int, 1>{});
                    // flags of the next iteration (its first byte belongs to the batch after this iteration's last)
                    const int itn = it + 1 < n_iter ? it + 1 : it;
                    const uint32_t fwn =
                        itn < kWave ? __builtin_amdgcn_readlane(fwv0, itn) : __builtin_amdgcn_readlane(fwv1, itn - kWave);
#pragma unroll
                    for (int j = 0; j < kRing; ++j) {
                        load_from(ring[(j + kRing - 1) % kRing], rp);
                        if (j == 0 && it + 1 == n_iter) rp = rp0;   // that was the part's last batch
                        else rp += 2 * kWave;
                        __builtin_amdgcn_sched_barrier(0);
                        fold(std::false_type{}, (fw >> (8 * j)) & 0xffu, ring[j], g[(NRES + j) % GB], g[(NRES + j + 1) % GB], ring[(j + 1) % kRing], false,
                             j + 1 < kRing || it + 1 < n_iter);
                    }
                    fw = fwn;
                }
                put_max(i, wmax);
                __syncthreads();
            };
            if constexpr (XF != 0) {
                for (int i = 1; i < Tn; i += 2) {
                    step(i, std::integral_constant<int, 0>{});
                    if (i + 1 < Tn) step(i + 1, std::integral_constant<int, 1>{});
                }
            } else {
                for (int i = 1; i < Tn; ++i) step(i, (i - 1) & 1);
            }
        }

        // ---- last frame: write it out, close log Z with the end weights
        const int last = (Tn - 1) & 1;
        const T *xl = xb + last * Xs;
        if (io_wave) write_row(frame(Tn - 1), bwd ? bh + last * Xs : xl);
        if (TROP) {
            if (io_wave && Tn >= 2) write_bp(Tn - 1, bpb + last * Xs);
            // score = max_k (x[k] + end weight) and a state that attains it (the smallest such k)
            T m = kNegInf;
            int at = 0x7fffffff;
            for (int k = tid; k < K; k += NT) {
                const T t = xl[k] + (T)R.obound[k0 + k];
                if (t > m) { m = t; at = k; }
            }
            for (int j = tid; j < sd.n_cdesc; j += NT) {   // clones end with their state's weight
                const CloneDesc cd = cdesc[j];
                for (int i = 0; i < cd.count; ++i) {
                    const T t = xl[P.Kcap + cd.first + i] + (T)R.obound[k0 + cd.state];
                    if (t > m || (t == m && P.Kcap + cd.first + i < at)) { m = t; at = P.Kcap + cd.first + i; }
                }
            }
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) {
                const T m2 = (T)__shfl_xor(m, o, 64);
                const int a2 = __shfl_xor(at, o, 64);
                if (m2 > m || (m2 == m && a2 < at)) { m = m2; at = a2; }
            }
            T *rm = red + 2 * NW, *rs = rm + NW;
            if (lane == 0) { rm[wave] = m; rs[wave] = (T)at; }
            __syncthreads();
            if (io_wave && lane == 0) {   // the lane that holds the sum of the offsets
                m = rm[0]; T a = rs[0];
                for (int w = 1; w < NW; ++w)
                    if (rm[w] > m || (rm[w] == m && rs[w] < a)) { m = rm[w]; a = rs[w]; }
                if (R.logz) R.logz[b] = (csum + (double)m) * kLn2;
                if (R.last) R.last[b] = m == kNegInf ? -1 : (int)a;
            }
        } else if (R.logz) {
            T m = (T)kNegBig;
            float s = 0.0f;
            for (int k = tid; k < K; k += NT) lse_add(m, s, xl[k] + (T)R.obound[k0 + k]);
            for (int j = tid; j < sd.n_cdesc; j += NT) {   // clones end with their state's weight
                const CloneDesc cd = cdesc[j];
                for (int i = 0; i < cd.count; ++i) lse_add(m, s, xl[P.Kcap + cd.first + i] + (T)R.obound[k0 + cd.state]);
            }
#pragma unroll
            for (int o = 32; o >= 1; o >>= 1) lse_merge(m, s, (T)__shfl_xor(m, o, 64), __shfl_xor(s, o, 64));
            T *rm = red + 2 * NW, *rs = rm + NW;
            if (lane == 0) { rm[wave] = m; rs[wave] = (T)s; }
            __syncthreads();
            if (io_wave && lane == 0) {   // the lane that holds the sum of the offsets
                m = rm[0]; s = (float)rs[0];
                for (int w = 1; w < NW; ++w) lse_merge(m, s, rm[w], (float)rs[w]);
                R.logz[b] = (csum + (double)m + (double)flog2(s)) * kLn2;
            }
        }
    } else if (tid == 0) {
        if (R.logz) R.logz[b] = -INFINITY;
        if (TROP && R.last) R.last[b] = -1;
    }

    // ---- padded frames
    if (R.fill_pad) {
        if (out_f)
            for (int f = Tn; f < P.N; ++f) {
                float *orow = out_f + (size_t)f * out_ld;
                for (int k = tid; k < K; k += NT) orow[k] = -INFINITY;
            }
        if (off_seq)
            for (int f = Tn + tid; f < P.N; f += NT) off_seq[f] = 0.0;
    }

}

// ---------------------------------------------------------------------------
// The same recursions carried in the probability domain (the matrix products of Eq. 4-5, rescaled at every step;
// the results handed out are those of Eq. 13-14).  For large shared graphs with float vectors.
//
// The vector in LDS holds P[k] = 2^(log2 of the true value - offset), the offset accumulated per sequence, so an
// arc costs one LDS gather and one multiply-add (the plan carries 2^w) and a row one exponential (its emission)
// instead of one exponential per arc.  At every step the vector is rescaled by the power of two that brings the
// previous step's largest entry to [2^bias, 2^(bias + 1)) (exact), and the emissions of a frame enter relative to
// the frame's largest emission over all pdfs (any scale serves).  bias is chosen per graph and direction so that no
// row sum can overflow (from the largest sum of weights of a row).
//
// The plan (fb_pstream.cpp).  Each arc-walking wave has a list of units - two arcs per lane in three registers - most
// of which stay in registers for the whole time loop (the rest cycles through a small ring fed from L2), a bit per
// unit that says whether a slice of rows ends there, and a register per slice that says, per lane, where the
// lane's sum goes and which emission it takes.  The order of the arcs in a lane and of the rows in a slice has been
// chosen on the host so that the 32 lanes of half a wave gather from different banks.
//
// Range guard.  A float holds what lies within 2^-126 of the scale; the log form holds everything.  An entry that is
// not the semiring zero must not come to lie below `dim`, the value under which its product with the graph's smallest
// weight could be flushed to zero.  A lane keeps the smallest entry it has written in a step for a row whose sum is
// above zero (an entry that an emission factor too small for a float has turned into zero included); if that is
// below `dim`, or if the step's largest entry falls too far for the next rescaling to be a float, the workgroup gives
// the sequence up (returns false) and its caller runs it again from the first frame in the log form.  Every sum a
// completed run has formed is therefore exact to rounding.  The give-up travels through the step maximum the waves
// exchange anyway: a lane that sees such a state reports +inf as its maximum.
//
// What leaves the kernel: the vectors as they are kept (RecDir::out_linear, for the gradient kernel) or, in the
// form of the other kernel, normalised rows as logarithms (the wave that closes a row stages its logarithm; the
// data-moving wave copies rows out either way); shifts and log Z as there.
// LDS: xb, the previous / current vector, kXsFixed floats each at addresses 0 and kXbStride; bh 2 x kXsFixed behind
// them (rows on their way out that are not the vector itself: beta before the emission is applied, or either
// direction's rows as logarithms; absent otherwise); red 64 floats (0-2 step maxima, 4-6 the frames' emission maxima
// in log2 units, 3 and 7 scratch of the first frame, 32-63 the last reduction); er 3 x Es floats, Es = D + 1
// rounded up to 4: the emissions as given of the frame in use and of the next two, entry D = -inf (what the dump
// slot "emits").
// ---------------------------------------------------------------------------
__device__ unsigned int g_linear_restarts;   // diagnostic: sequences (x directions) given up by linear_run since the library was loaded

typedef uint32_t close_vector_t __attribute__((ext_vector_type(2 * kPMaxClose)));

__device__ __forceinline__ bool linear_run(const RecParams &P, const int b, const int which, double *lds_raw)
{
    constexpr int NW = kNWShared, XF = kXsFixed, R = kPResident;
    constexpr int NT = NW * kWave, NC = NW - 1;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool io_wave = wave == NC;
    const RecDir &R_ = P.dir[which];
    const PStreamDev &S = R_.prob;
    const bool bwd = R_.backward != 0;
    const int K = P.Kcap, nC = S.Ccap;
    const int Tn = min(max(P.lengths[b], 0), P.N);
    const int nE = P.D;
    const int nX = K + nC + 1;                   // states, clone slots, dump slot
    // the two buffers of the vector in use lie kXbStride bytes apart, further than a buffer is long and a power of two:
    // an arc's source (an offset into a buffer) and the buffer's address then combine by OR
    constexpr int Xs = kXbStride / 4;
    static_assert(kXbStride >= XF * 4 && (kXbStride & (kXbStride - 1)) == 0 && 2 * kXbStride <= 0x10000, "buffer stride");
    const int Es = (P.D + 1 + 3) & ~3;
    if (Tn <= 0) return false;                   // (nothing to run: the log form writes the empty results)

    float *xb = (float *)lds_raw;
    // rows on their way out that are not the vector itself: beta before the emissions are applied (backward), and
    // either direction's rows as logarithms when that is the form they leave in; two buffers that follow each other,
    // present only when used
    const bool log_rows = R_.out != nullptr && R_.out_linear == 0;
    const bool staged = bwd || log_rows;
    float *bh = xb + Xs + XF;
    float *red = staged ? bh + 2 * XF : bh;
    float *er = red + 64;
    float *emaxw = red + 4;

    const float *em_seq = P.emis + (size_t)b * P.N * P.D;
    const size_t out_ld = (size_t)(R_.out_ld ? R_.out_ld : K);
    float *out_row0 = R_.out ? (float *)R_.out + (size_t)b * P.N * out_ld : nullptr;
    double *off_seq = R_.off ? R_.off + (size_t)b * P.N : nullptr;
    auto frame = [&](int i) { return bwd ? Tn - 1 - i : i; };
    auto put_max = [&](int i, float wmax) {
        wmax = wave_max(wmax);
        if (lane == 0) __builtin_amdgcn_ds_fmaxf((__attribute__((address_space(3))) float *)(red + i % 3), wmax, 0, 0, false);
    };
    const int kLinBias = S.bias;
    const float kLinDimP = S.dim;
    const float unbias = __uint_as_float((uint32_t)(127 - kLinBias) << 23);   // 2^-bias
    // a step maximum the run cannot go on from: a lane gave up (+inf), or the vector fell more than 126 binary orders
    // in one step (its rescaling would not be a float)
    const float mx_floor = __uint_as_float((uint32_t)max(kLinBias - 126 + 127, 1) << 23);
    auto gives_up = [&](float mx) { return !(mx < INFINITY) || (mx > 0.0f && mx < mx_floor); };
    // the power of two that brings mx (finite, 0 or >= mx_floor) to [2^bias, 2^(bias + 1)), and minus its log2
    auto rescale = [&](float mx, float &sc, float &neg_log2_sc) {
        const int ex = (int)((__float_as_uint(mx) >> 23) & 0xffu);
        const bool live = mx > 0.0f;
        sc = live ? __uint_as_float((uint32_t)(254 + kLinBias - ex) << 23) : 1.0f;
        neg_log2_sc = live ? (float)(ex - 127 - kLinBias) : 0.0f;
    };

    // ---- duties of the data-moving wave
    // a frame's emissions -> LDS, 16 bytes a lane where the row allows it; the lane's address is formed once and every
    // piece but the last is loaded by all lanes
    auto stage = [&](int f, float *dst) {
        const float *row = em_seq + (size_t)f * P.D;
        typedef const __attribute__((address_space(1))) void gvoid;
        typedef __attribute__((address_space(3))) void lvoid;
        if ((P.D & 3) == 0 && ((uintptr_t)row & 15) == 0) {
            const float *mine = row + 4 * lane;
            int e0 = 0;
            for (; e0 + 4 * kWave <= nE; e0 += 4 * kWave) __builtin_amdgcn_global_load_lds((gvoid *)(mine + e0), (lvoid *)(dst + e0), 16, 0, 0);
            if (e0 + 4 * lane < nE) __builtin_amdgcn_global_load_lds((gvoid *)(mine + e0), (lvoid *)(dst + e0), 16, 0, 0);
        } else {
            const float *mine = row + lane;
            int e0 = 0;
            for (; e0 + kWave <= nE; e0 += kWave) __builtin_amdgcn_global_load_lds((gvoid *)(mine + e0), (lvoid *)(dst + e0), 4, 0, 0);
            if (e0 + lane < nE) __builtin_amdgcn_global_load_lds((gvoid *)(mine + e0), (lvoid *)(dst + e0), 4, 0, 0);
        }
    };
    auto staged_wait = [&]() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); };
    // The largest emission of a staged frame, in log2 units (0 if there is none above zero-bar).  Over all pdfs, whether
    // a state of the graph is tied to them or not: any scale serves.  16 bytes per lane and read (the arc-walking waves
    // keep the LDS queue full: few, wide reads); what lies behind the row in its last group is -inf.
    auto emax_of = [&](const float *row) {
        float m = -INFINITY;
        const float4 *r4 = (const float4 *)row;
        const int n4e = Es / 4;
        constexpr int U = 8;
        for (int j0 = 0; j0 * kWave < n4e; j0 += U) {
            float4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = r4[min((j0 + u) * kWave + lane, n4e - 1)];
#pragma unroll
            for (int u = 0; u < U; ++u) m = tmax3(tmax3(m, v[u].x, v[u].y), v[u].z, v[u].w);
        }
        m = wave_max(m) * (float)kLog2e;
        return m > -INFINITY ? m : 0.0f;
    };
    const CloneDesc *cdesc = S.clones;
    // a finished vector -> global memory, coalesced; a cloned state leaves as the sum of its clones.  Either as it is
    // (RecDir::out_linear: the reader has the offsets and the scale) or as log2 of (entry x 2^-bias) x out_scale, the
    // exponent and the mantissa taken apart first so that neither an entry far below the scale is lost nor the
    // entries near it are rounded at the magnitude of the bias.
    const bool out_lin = R_.out_linear != 0;
    auto to_log = [&](float v) {
        const float e = (float)(__builtin_amdgcn_frexp_expf(v) - kLinBias);   // (v = 0: -inf comes from the mantissa)
        return (e + flog2(__builtin_amdgcn_frexp_mantf(v))) * R_.out_scale;
    };
    // (rows that leave as logarithms were staged in that form by the waves that formed them: a plain copy either way)
    auto write_row = [&](int f, const float *srcv) {
        if (!out_row0) return;
        float *orow = out_row0 + (size_t)f * out_ld;
        const float4 *s4 = (const float4 *)srcv;
        const int n4 = (K + 3) / 4;
        const bool vec = (out_ld & 3) == 0 && (size_t)(n4 * 4) <= out_ld && ((uintptr_t)orow & 15) == 0;
        constexpr int U = 8;
        for (int q0 = 0; q0 < n4; q0 += U * kWave) {
            float4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) v[u] = s4[min(q0 + u * kWave + lane, n4 - 1)];
#pragma unroll
            for (int u = 0; u < U; ++u)   // every read and conversion stays in front of the stores
                asm volatile("" : "+v"(v[u].x), "+v"(v[u].y), "+v"(v[u].z), "+v"(v[u].w));
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int q = q0 + u * kWave + lane;
                if (q < n4) {
                    if (vec) {   // (the row's padding may take up to 3 values that lie behind the states)
                        // (a streaming store: the row is read again much later, by another kernel, and what it would
                        // push out of L2 is the arc plan every workgroup re-reads at every step)
                        typedef float f4 __attribute__((ext_vector_type(4)));
                        const f4 t = {v[u].x, v[u].y, v[u].z, v[u].w};
                        __builtin_nontemporal_store(t, (f4 *)orow + q);
                    } else {
                        if (4 * q + 0 < K) orow[4 * q + 0] = v[u].x;
                        if (4 * q + 1 < K) orow[4 * q + 1] = v[u].y;
                        if (4 * q + 2 < K) orow[4 * q + 2] = v[u].z;
                        if (4 * q + 3 < K) orow[4 * q + 3] = v[u].w;
                    }
                }
            }
        }
        for (int j = lane; j < S.n_clones; j += kWave) {   // stores of one wave to one address keep their order
            const CloneDesc cd = cdesc[j];
            if (out_lin) {
                float t = srcv[cd.state];
                for (int i = 0; i < cd.count; ++i) t += srcv[K + cd.first + i];
                orow[cd.state] = t;
            } else {   // logarithms (scaled by out_scale, which is positive): the (+)-sum of the clones
                float m = srcv[cd.state];
                for (int i = 0; i < cd.count; ++i) m = tmax(m, srcv[K + cd.first + i]);
                float t = 0.0f;
                if (m > -INFINITY) {
                    const float inv = 1.0f / R_.out_scale;
                    t = fexp2((srcv[cd.state] - m) * inv);
                    for (int i = 0; i < cd.count; ++i) t += fexp2((srcv[K + cd.first + i] - m) * inv);
                }
                orow[cd.state] = m > -INFINITY ? m + flog2(t) * R_.out_scale : m;
            }
        }
    };
    // what the readers of a row get beside it: log2 of the true row = log2 of the stored row + cum (in the linear
    // form the stored row still carries the scale 2^bias)
    const double cum_shift = out_lin ? (double)kLinBias : 0.0;

    // ---- first frame of this direction: the start weights and the frame's emissions, relative to their maximum
    if (tid < 12) er[(tid >> 2) * Es + Es - 4 + (tid & 3)] = -INFINITY;   // behind the rows (staging never writes there; the row's own last entries are rewritten)
    __syncthreads();
    if (tid < 3) er[tid * Es + P.D] = -INFINITY;   // what the dump slot "emits": its entry stays zero whatever the frame's scale
    if (tid < 8) red[tid] = (tid == 7 || tid == 3) ? -INFINITY : 0.0f;
    __syncthreads();
    if (io_wave) {
        stage(frame(0), er);
        if (Tn > 1) stage(frame(1), er + Es);
        staged_wait();
        const float e0 = emax_of(er);
        const float e1 = Tn > 1 ? emax_of(er + Es) : 0.0f;
        if (lane == 0) { emaxw[0] = e0; emaxw[1] = e1; }
        if (Tn > 2) stage(frame(2), er + 2 * Es);   // lands while step 1 runs
    }
    __syncthreads();
    const float emx0 = emaxw[0];
    {
        float ymax = -INFINITY, smax = -INFINITY;
        for (int k = tid; k < K; k += NT) {
            const float s = R_.bound[k];
            ymax = tmax(ymax, s + fmaf(er[P.pdf[k]], (float)kLog2e, -emx0));
            smax = tmax(smax, s);
        }
        ymax = wave_max(ymax);
        smax = wave_max(smax);
        if (lane == 0) {
            __builtin_amdgcn_ds_fmaxf((__attribute__((address_space(3))) float *)(red + 7), ymax, 0, 0, false);
            __builtin_amdgcn_ds_fmaxf((__attribute__((address_space(3))) float *)(red + 3), smax, 0, 0, false);
        }
    }
    __syncthreads();
    const float M0 = red[7];
    // log2 of the first vector = log2 of its entries + base0 (+ the emission maximum).  The largest entry goes to
    // 2^bias; backward, the row that leaves is the start weights before the frame's emissions, which lie above the
    // vector by what the best state's emission lacks to the frame's largest: the scale is held back as far as that
    // row needs to stay a float (the vector's entries are then smaller, and below the range the run gives up as ever).
    float base0 = M0 > -INFINITY ? M0 - (float)kLinBias : 0.0f;
    if (bwd && M0 > -INFINITY) base0 = tmax(base0, red[3] - 126.0f);
    float wmax = 0.0f;
    for (int k = tid; k < K; k += NT) {
        const float s = R_.bound[k];
        const float y = s + fmaf(er[P.pdf[k]], (float)kLog2e, -emx0) - base0;
        const float px = fexp2(y);
        xb[k] = px;
        if (log_rows) bh[k] = ((bwd ? s - base0 : y) - (float)kLinBias) * R_.out_scale;
        else if (bwd) bh[k] = fexp2(s - base0);
        const bool dim = y > -INFINITY && px < kLinDimP;
        wmax = dim ? INFINITY : tmax(wmax, px);
    }
    for (int k = tid; k < nC; k += NT) {   // clones start empty: the state itself holds the start weight
        xb[K + k] = 0.0f;
        if (staged) bh[K + k] = log_rows ? -INFINITY : 0.0f;
    }
    if (tid == 0) xb[nX - 1] = xb[Xs + nX - 1] = 0.0f;   // the dump slot holds zero in both buffers, always
    put_max(0, wmax);
    __syncthreads();

    // offsets: log2 of the true row of step i = log2 of (the row in LDS x 2^-bias: what is written out) + sum_{j <= i} c_j,
    // with c_0 = base0 + bias (+ the emission maximum of the frame, forward) and c_i = -log2(scale of step i) + the
    // emission maximum of frame(i) (forward) or of frame(i - 1) (backward: the row sum of Eq. 14 is taken before the
    // frame's own emission)
    double csum = 0.0;
    bool ok = true;
    if (io_wave) {
        float c = base0 + (float)kLinBias + (bwd ? 0.0f : emx0);
        csum = (double)c;
        if (lane == 0) {
            if (off_seq) off_seq[frame(0)] = csum * (double)R_.out_scale;
            if (R_.cum) R_.cum[(size_t)b * P.N + frame(0)] = (float)(csum - cum_shift);
        }
        for (int i = 1; i < Tn; ++i) {
            const int cur = (i - 1) & 1;
            const float mx = red[(i - 1) % 3];
            if (gives_up(mx)) { ok = false; break; }
            float sc, nls;
            rescale(mx, sc, nls);
            c = nls + emaxw[(bwd ? i - 1 : i) % 3];
            csum += (double)c;
            if (lane == 0) {
                if (off_seq) off_seq[frame(i)] = csum * (double)R_.out_scale;
                if (R_.cum) R_.cum[(size_t)b * P.N + frame(i)] = (float)(csum - cum_shift);
            }
            staged_wait();   // frame i+1, requested a whole step ago, is in LDS
            if (i + 1 < Tn) {
                const float en = emax_of(er + ((i + 1) % 3) * Es);
                if (lane == 0) emaxw[(i + 1) % 3] = en;   // (the word of frame i - 2: read for the last time in step i - 1)
            }
            if (i + 2 < Tn) stage(frame(i + 2), er + ((i + 2) % 3) * Es);   // buffer of frame i-1: no longer read
            write_row(frame(i - 1), staged ? bh + cur * XF : xb + cur * Xs);
            if (lane == 0) red[(i + 1) % 3] = 0.0f;   // the word of step i + 1 starts empty
            __syncthreads();
        }
    } else {
        const PWaveDesc wd = S.waves[wave];
        const int n_units_w = __builtin_amdgcn_readfirstlane(wd.n_units);
        auto uniform64 = [](uint64_t v) {
            return (uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v) |
                   ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32)) << 32);
        };
        const uint64_t mask0_w = uniform64(wd.close_mask[0]), mask1_w = uniform64(wd.close_mask[1]), lgs_w = uniform64(wd.lgs);
        struct Unit { uint32_t s; float w0, w1; };
        // unit u of the wave: a wave-uniform base (three words per lane) plus the lane's 12 bytes
        const uint32_t *const ubase = S.units + (size_t)uniform64((uint64_t)wd.unit_base) * (3 * kWave);
        const uint32_t lane3 = (uint32_t)lane * 3u;
        auto load_unit = [&](Unit &dst, const uint32_t *base) __attribute__((always_inline)) {
            dst.s = base[lane3];
            dst.w0 = __uint_as_float(base[lane3 + 1]);
            dst.w1 = __uint_as_float(base[lane3 + 2]);
        };
        // The wave's units in walking order (see kPPatterned): which positions stay in registers, which are re-read.
        // Re-read ("streamed") unit m of a step sits in ring[m % kPRing] and is asked for kPRing - 1 streamed units ahead
        // of its use; the first kPRing - 1 of a step when the step before ends.  Every place that asks does so whatever
        // the wave's unit count (for a unit that is not there, the last one again): the number of loads on their way
        // at any point of the code is then a constant, which is what the waits on them are counted by.
        constexpr int NP = kPPatterned, H = kPHead, NG = NP - R;   // patterned positions, head, re-read ones among them
        static_assert(NP <= 64 && NP % 16 == 0 && NG >= kPRing - 1, "close bits of the patterned part in one 64-bit word; blocks of 4, a priority level for every quarter");
        // the position of the wave's last re-read unit: what a request for a unit behind it asks for again (a wave
        // without any asks for a unit behind its own: never folded, and the plan has room behind every wave)
        int last_spos = p_streamed_pos(0);
        unrolled([&](auto uc) __attribute__((always_inline)) {
            constexpr int u = decltype(uc)::value;
            if constexpr (p_streamed(u)) last_spos = u < n_units_w ? u : last_spos;
        }, std::make_integer_sequence<int, NP>{});
        if (n_units_w > NP) last_spos = n_units_w - 1;
        Unit res[R];   // (units behind the wave's last one are zero words or another wave's: never folded)
        unrolled([&](auto qc) __attribute__((always_inline)) {
            constexpr int q = decltype(qc)::value;
            load_unit(res[q], ubase + (size_t)p_resident_pos(q) * (3 * kWave));
        }, std::make_integer_sequence<int, R>{});
        // The lane's close words and, behind them, the emission factors of the step in hand, both picked by the number
        // of the close (uniform).  One vector of sixteen: picking from a vector of eight is compiled into a chain of seven
        // selects, from a longer one into one indexed register move.
        close_vector_t cwv;
#pragma unroll
        for (int c = 0; c < kPMaxClose; ++c) cwv[c] = S.close_words[((size_t)wd.cw_base + c) * kWave + lane];
        // (everything asked for so far has arrived: the waits inside the loop then count the loop's own loads only)
        __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0)
        Unit ring[kPRing];
        // streamed unit m -> its ring place (in the patterned part streamed unit m is position H + 3 m + 2; behind it, unit
        // NP + t is streamed unit NG + t)
        // (the base the requests add to is made opaque at every step: an address formed at the place of the request is a
        // scalar base plus the lane's offset, while addresses kept over the whole loop, as the compiler would have them,
        // take a register pair each)
        uint32_t ub_lo = (uint32_t)(uintptr_t)ubase, ub_hi = (uint32_t)((uintptr_t)ubase >> 32);
        // (a position inside the patterned part is asked for as it is, whatever the wave's unit count: the plan has
        // room for kPPatterned units behind every wave's first; positions behind it are held to the wave's last unit)
        auto request_at = [&](Unit &dst, int u) __attribute__((always_inline)) {
            typedef const __attribute__((address_space(1))) uint32_t global_u32;   // (an address built from integers: say that it is global memory)
            global_u32 *ub = (global_u32 *)((uintptr_t)ub_lo | ((uintptr_t)ub_hi << 32)) + (size_t)u * (3 * kWave);
            dst.s = ub[lane3];
            dst.w0 = __uint_as_float(ub[lane3 + 1]);
            dst.w1 = __uint_as_float(ub[lane3 + 2]);
            __builtin_amdgcn_sched_barrier(0);   // keep the issue order: waits count loads in order
        };
        auto request = [&](Unit &dst, int pos) __attribute__((always_inline)) { request_at(dst, min(pos, last_spos)); };
        unrolled([&](auto mc) __attribute__((always_inline)) {
            constexpr int m = decltype(mc)::value;
            request_at(ring[m], p_streamed_pos(m));
        }, std::make_integer_sequence<int, kPRing - 1>{});

        auto step = [&](int i) __attribute__((always_inline)) -> bool {
            const int cur = (i - 1) & 1, nxt = cur ^ 1;   // which buffer holds the previous step's vector
            float *xn = xb + nxt * Xs;
            float *bn = bh + nxt * XF;
            const uint32_t gbase = (uint32_t)cur * (uint32_t)kXbStride;   // (uniform) address of the buffer the gathers read
            const char *ern = (const char *)(er + (i % 3) * Es);
            const float mx = red[(i - 1) % 3];
            if (gives_up(mx)) return false;   // (the same word in every wave: all of them leave here)
            float sc, nls;
            rescale(mx, sc, nls);
            const float emx = emaxw[i % 3];
            wmax = 0.0f;
            // the smallest entry this lane has written for a row whose sum is above zero, as its bit pattern (which keeps
            // the order of floats that are not negative)
            uint32_t wlow = 0x7f800000u;
            float acc = 0.0f;
            // the wave's constants, opaque at every step: what is derived from them is computed where it is used (a
            // scalar instruction or two) instead of being kept in scalar registers that do not exist
            uint32_t m_lo = (uint32_t)mask0_w, m_hi = (uint32_t)(mask0_w >> 32), m1_lo = (uint32_t)mask1_w, m1_hi = (uint32_t)(mask1_w >> 32);
            uint32_t lg_lo = (uint32_t)lgs_w;
            int n_units = n_units_w;
            asm volatile("" : "+s"(m_lo), "+s"(m_hi), "+s"(m1_lo), "+s"(m1_hi), "+s"(lg_lo), "+s"(n_units), "+s"(ub_lo), "+s"(ub_hi), "+s"(last_spos));
            int nclose = 0;   // slices closed so far in this step (uniform)
            if (i <= 2)   // rows without arcs: zero from the second frame on, in both buffers
                for (int z = tid; z < S.n_zero; z += NC * kWave) {
                    const int k = S.zero_rows[z];
                    xn[k] = 0.0f;
                    if (staged) bn[k] = log_rows ? -INFINITY : 0.0f;
                }
            // the two values a unit gathers; sources are byte offsets, the workgroup's LDS starts at address 0
            auto gather = [&](float2 &g, uint32_t s) __attribute__((always_inline)) {
                typedef const __attribute__((address_space(3))) float lds_ct;
                // one instruction per address: a half of the word, zero-extended, OR the buffer's address.  (In assembly
                // also so that the addresses are formed at every step: left to itself the compiler keeps every resident
                // unit's two addresses in registers of their own.)
                uint32_t lo, hi;
                asm volatile("v_or_b32_sdwa %0, %3, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_0\n\t"
                             "v_or_b32_sdwa %1, %3, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:WORD_1"
                             : "=&v"(lo), "=v"(hi) : "v"(s), "s"(gbase));
                g.x = *(lds_ct *)(uintptr_t)lo;
                g.y = *(lds_ct *)(uintptr_t)hi;
            };
            // a slice ends: the lanes of a row are added up, the row is rescaled, takes its emission, is stored.  The
            // emission of the slice that ends next is asked for as soon as the one before it has ended, so that it has
            // arrived when it is needed (LDS answers in order: asked for at the end, it would wait behind the gathers).
            // the emission factors of the wave's closes, relative to the frame's best: read and raised here, so that a
            // close waits for nothing but its own arcs
            typedef const __attribute__((address_space(3))) float lds_cf;
            const uint32_t ern_a = (uint32_t)(uintptr_t)ern;
#pragma unroll
            for (int c = 0; c < kPMaxClose; ++c)
                cwv[kPMaxClose + c] = __float_as_uint(fexp2(fmaf(*(lds_cf *)(uintptr_t)(ern_a + (cwv[c] >> 16)), (float)kLog2e, -emx)));
            // a slice ends: the lanes of a row are added up, the row is rescaled, takes its emission, is stored
            auto close_slice = [&]() __attribute__((always_inline)) {
                const int lg = (int)((lg_lo >> (3 * nclose)) & 7u);
                const uint32_t tgt = cwv[nclose] & 0xffffu;
                const float pe = __uint_as_float(cwv[kPMaxClose + nclose]);
                ++nclose;
                for (int sft = 0; sft < lg; ++sft)   // the lanes of a row are neighbours: a butterfly over 2^lg lanes (few rows are that long)
                    acc += __uint_as_float((uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ (1 << sft)) << 2, (int)__float_as_uint(acc)));
                const float pb = acc * sc;
                const float px = pb * pe;
                *(float *)((char *)xn + tgt) = px;
                if (staged) {   // (uniform) what leaves the kernel for this row
                    const float o = bwd ? pb : px;
                    *(float *)((char *)bn + tgt) = log_rows ? to_log(o) : o;
                }
                wmax = tmax(wmax, px);
                wlow = min(wlow, __float_as_uint(pb > 0.0f ? px : INFINITY));
                acc = 0.0f;
            };
            // position u of the patterned part: which registers hold it
            auto unit_at = [&](auto uc) __attribute__((always_inline)) -> Unit {
                constexpr int u = decltype(uc)::value;
                if constexpr (p_streamed(u)) return ring[p_streamed_before(u) % kPRing];
                else return res[u - p_streamed_before(u)];
            };
            // gathered values of the unit being folded and of the next GD: under load a gather takes a few hundred cycles
            constexpr int GD = 3, NGB = GD + 1;
            static_assert(kPRing % NGB == 0 && NG % kPRing == 0 && GD <= H && GD <= kPRing - 1, "buffer names repeat with the ring; the first gathers are of resident units");
            float2 G[NGB];
            unrolled([&](auto uc) __attribute__((always_inline)) {
                constexpr int u = decltype(uc)::value;
                gather(G[u], unit_at(std::integral_constant<int, u>{}).s);
            }, std::make_integer_sequence<int, GD>{});
            // Waves of equal priority are served oldest first, so with one fixed priority the younger waves of a SIMD
            // would do most of their step alone after the older ones have finished theirs.  A wave's priority therefore
            // falls as its step advances, a level for every quarter: whoever has more left goes first.
            __builtin_amdgcn_s_setprio(3);
            // (the units are in order, so nothing follows a unit that is not there; looked at every fourth position)
            auto block = [&](auto self, auto kc) __attribute__((always_inline)) -> void {
                constexpr int u0 = decltype(kc)::value * 4;
                if constexpr (u0 < NP) {
                    if (n_units > u0) {
                        if constexpr (u0 % (NP / 4) == 0 && u0 > 0) __builtin_amdgcn_s_setprio(3 - u0 / (NP / 4));
                        unrolled([&](auto jc) __attribute__((always_inline)) {
                            constexpr int u = u0 + decltype(jc)::value;
                            // a streamed unit: the place of the one before it in the ring is free, the unit kPRing - 1 further on goes there
                            if constexpr (p_streamed(u)) {
                                constexpr int m = p_streamed_before(u);
                                if constexpr (p_streamed_pos(m + kPRing - 1) < NP) request_at(ring[(m + kPRing - 1) % kPRing], p_streamed_pos(m + kPRing - 1));
                                else request(ring[(m + kPRing - 1) % kPRing], p_streamed_pos(m + kPRing - 1));
                            }
                            // (gathered whether the wave has that unit or not - its registers hold valid sources either way -
                            // so that the number of gathers on their way is a constant too)
                            if constexpr (u + GD < NP) gather(G[(u + GD) % NGB], unit_at(std::integral_constant<int, u + GD>{}).s);
                            else gather(G[(u + GD) % NGB], ring[(NG + (u + GD - NP)) % kPRing].s);   // the first units behind the patterned part
                            const Unit me = unit_at(std::integral_constant<int, u>{});
                            // (both values of the unit are taken at one point: one wait for the pair instead of one each)
                            asm volatile("" : "+v"(G[u % NGB].x), "+v"(G[u % NGB].y));
                            acc = fmaf(G[u % NGB].x, me.w0, acc);
                            acc = fmaf(G[u % NGB].y, me.w1, acc);
                            if (((u < 32 ? m_lo : m_hi) >> (u & 31)) & 1u) close_slice();
                        }, std::make_integer_sequence<int, 4>{});
                        self(self, std::integral_constant<int, decltype(kc)::value + 1>{});
                    }
                }
            };
            block(block, std::integral_constant<int, 0>{});
            // behind the patterned part: streamed units; unit NP + t is streamed unit NG + t; kPRing positions to a round,
            // so that the names of the ring places and of the gather buffers repeat
            static_assert(NP % NGB == 0 && NG % kPRing != -1, "rounds");
            for (int t0 = 0; NP + t0 < n_units; t0 += kPRing) {
#pragma unroll
                for (int tt = 0; tt < kPRing; ++tt) {   // (a plain loop: closures inside a loop that stays a loop are not taken apart by the compiler)
                    const int t = t0 + tt;
                    if (NP + t < n_units) {
                        const int mr = NG + tt;   // (t0 is a multiple of kPRing: only tt names the buffers)
                        request(ring[(mr + kPRing - 1) % kPRing], NP + t + kPRing - 1);
                        gather(G[(NP + tt + GD) % NGB], ring[(mr + GD) % kPRing].s);
                        asm volatile("" : "+v"(G[(NP + tt) % NGB].x), "+v"(G[(NP + tt) % NGB].y));
                        acc = fmaf(G[(NP + tt) % NGB].x, ring[mr % kPRing].w0, acc);
                        acc = fmaf(G[(NP + tt) % NGB].y, ring[mr % kPRing].w1, acc);
                        const int at = NP + t;
                        const uint32_t word = at < 32 ? m_lo : at < 64 ? m_hi : at < 96 ? m1_lo : m1_hi;
                        if ((word >> (at & 31)) & 1u) close_slice();
                    }
                }
            }
            // the first streamed units of the next step (every place of the ring is free now)
            unrolled([&](auto mc) __attribute__((always_inline)) {
                constexpr int m = decltype(mc)::value;
                request_at(ring[m], p_streamed_pos(m));
            }, std::make_integer_sequence<int, kPRing - 1>{});
            // an entry below the range: the run gives up (see above)
            const bool low = wlow < __float_as_uint(kLinDimP);
            put_max(i, low ? INFINITY : wmax);
            __syncthreads();
            return true;
        };
        for (int i = 1; i < Tn && ok; ++i) ok = step(i);
    }
    // a state below the range in the last step: give up as well (every wave reads the same word)
    if (ok && !(red[(Tn - 1) % 3] < INFINITY)) ok = false;   // (the last vector is not rescaled: only a lane's give-up counts)
    __builtin_amdgcn_s_setprio(3);
    if (!ok) {
        // every wave has left the time loop at the same step; nothing of this run may still be on its way to LDS or
        // to the output rows when the log form starts over
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) atomicAdd(&g_linear_restarts, 1u);
        return false;
    }

    // ---- last frame: write it out, close log Z with the end weights
    const int last = (Tn - 1) & 1;
    const float *xl = xb + last * Xs;
    if (io_wave) write_row(frame(Tn - 1), staged ? bh + last * XF : xl);
    if (R_.logz) {
        float m = kNegBig, s = 0.0f;
        for (int k = tid; k < K; k += NT) lse_add(m, s, flog2(xl[k] * unbias) + R_.obound[k]);
        for (int j = tid; j < S.n_clones; j += NT) {   // clones end with their state's weight
            const CloneDesc cd = cdesc[j];
            for (int i = 0; i < cd.count; ++i) lse_add(m, s, flog2(xl[K + cd.first + i] * unbias) + R_.obound[cd.state]);
        }
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) lse_merge(m, s, __shfl_xor(m, o, 64), __shfl_xor(s, o, 64));
        float *rm = red + 32, *rs = rm + NW;
        const float em_last = emaxw[(Tn - 1) % 3];
        if (lane == 0) { rm[wave] = m; rs[wave] = s; }
        __syncthreads();
        if (io_wave && lane == 0) {   // the lane that holds the sum of the offsets
            m = rm[0]; s = rs[0];
            for (int w = 1; w < NW; ++w) lse_merge(m, s, rm[w], rs[w]);
            // backward: the vector of the last step still lacks the scale of its frame's emissions
            R_.logz[b] = (csum + (bwd ? (double)em_last : 0.0) + (double)m + (double)flog2(s)) * kLn2;
        }
    }
    // ---- padded frames
    if (R_.fill_pad) {
        if (out_row0)
            for (int f = Tn; f < P.N; ++f) {
                float *orow = out_row0 + (size_t)f * out_ld;
                for (int k = tid; k < K; k += NT) orow[k] = -INFINITY;
            }
        if (off_seq)
            for (int f = Tn + tid; f < P.N; f += NT) off_seq[f] = 0.0;
    }
    if (R_.fmt && tid == 0) R_.fmt[b] = out_lin ? 1 : 0;   // which form this sequence's rows have
    return true;
}

__global__ __launch_bounds__(kNWShared * 64) void fb_linear_kernel(const RecParams P)
{
    __builtin_amdgcn_s_setprio(3);
    extern __shared__ double lds_raw[];
    int b, which;
    if (P.started && threadIdx.x == 0) atomicAdd(P.started, 1u);   // this workgroup has its compute unit
    resolve_sequence<kNWShared>(P, lds_raw, b, which);
    if (!linear_run(P, b, which, lds_raw)) {
        recursion_run<kNWShared, float, false, kXsFixed, false>(P, b, which, lds_raw);
        if (P.dir[which].fmt && threadIdx.x == 0) P.dir[which].fmt[b] = 0;   // this sequence's rows are in the log form
    }
    count_done(P);
}

template <int NW, class T, bool TROP, int XF, bool LINW = false>
__global__ __launch_bounds__(NW * 64) void fb_recursion_kernel(const RecParams P)
{
    // The large-graph kernel is the critical path of a call; small-graph launches that run beside it on the same
    // compute units (the numerators of an LF-MMI call) take the issue slots it leaves.  (The data-moving wave
    // keeps this priority; the others vary theirs within a time step.)
    if (NW == kNWShared) __builtin_amdgcn_s_setprio(3);
    extern __shared__ double lds_raw[];
    int b, which;
    if (P.started && threadIdx.x == 0) atomicAdd(P.started, 1u);   // this workgroup has its compute unit
    resolve_sequence<NW>(P, lds_raw, b, which);
    recursion_run<NW, T, TROP, XF, LINW>(P, b, which, lds_raw);
    count_done(P);
}

// ---------------------------------------------------------------------------
// Posteriors (Eq. 15) of one or two graphs and their accumulation into pdf
// posteriors; each graph enters with its sign (Eq. 17: numerator minus
// denominator).  grid = (ceil(N / frames_per_block), B), kPostThreads threads.
// A workgroup keeps the states-by-pdf tables of its sequence's graphs in LDS and
// walks its frames one at a time: log posteriors of the frame -> LDS, maximum,
// exponentials, sum, then one thread per pdf adds up the states tied to it in a
// fixed order (no atomics: results do not depend on timing).
// ---------------------------------------------------------------------------
constexpr int kPostThreads = 512;

namespace {

// First pass over one frame of one graph: log posteriors (a + b) * in_scale into stage[0..K); returns
// the thread's maximum.  IT: element type of a and b.
template <class IT>
__device__ __forceinline__ IT frame_logpost(const IT *arow, const IT *brow, IT in_scale, int K, IT *stage, int tid)
{
    IT mx = (IT)(-INFINITY);
    for (int k = tid; k < K; k += kPostThreads) {
        const IT t = (arow[k] + brow[k]) * in_scale;
        stage[k] = t;
        mx = tmax(mx, t);
    }
    return mx;
}

// Rest of the frame: block maximum, exp2(log posterior - max) into tb[0..K) (unnormalised); returns
// 1 / their sum (0 if the frame has no mass).  stage: tb itself, or a wider buffer.
template <class IT>
__device__ __forceinline__ float frame_finish(IT mx, int K, float *tb, const IT *stage, float *red, int tid, int lane, int wave)
{
    constexpr int NT = kPostThreads, NWV = kPostThreads / kWave;
    mx = wave_max(mx);
    IT *redt = (IT *)red;
    if (lane == 0) redt[wave] = mx;
    __syncthreads();
    mx = redt[0];
#pragma unroll
    for (int w = 1; w < NWV; ++w) mx = tmax(mx, redt[w]);
    __syncthreads();
    float sum = 0.0f;
    if (mx != (IT)(-INFINITY))
        for (int k = tid; k < K; k += NT) {
            const float e = fexp2((float)(stage[k] - mx));
            tb[k] = e;      // tb may alias stage when IT is float: same index, read before write
            sum += e;
        }
    else
        for (int k = tid; k < K; k += NT) tb[k] = 0.0f;
    sum = wave_sum(sum);
    if (lane == 0) red[wave] = sum;
    __syncthreads();
    sum = red[0];
#pragma unroll
    for (int w = 1; w < NWV; ++w) sum += red[w];
    return sum > 0.0f ? 1.0f / sum : 0.0f;
}

constexpr int kPostPrefetch = 3;   // 16-byte pieces per thread and array held in registers: 6144 states

}  // namespace

__global__ __launch_bounds__(kPostThreads) void fb_posterior_kernel(const PostParams P)
{
    extern __shared__ double lds_raw[];
    constexpr int NT = kPostThreads, U = kPostPrefetch;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int b = P.order ? P.order[P.rank0 + blockIdx.y] : blockIdx.y;
    const int T = min(max(P.lengths[b], 0), P.N);
    const int n0 = blockIdx.x * P.frames_per_block;
    const int n_end = min(min(n0 + P.frames_per_block, P.N), T);   // real frames of this chunk: [n0, n_end)
    float *red = (float *)lds_raw;                  // reduction slots: one double or float per wave
    double *stage64 = lds_raw + 8;                  // [Kcap64] log posteriors of a double-carrier graph
    float *tb = (float *)(stage64 + P.Kcap64);      // [Kcap] per-state values of the frame
    float *rho = tb + P.Kcap;                       // [D]
    uint16_t *tab = (uint16_t *)(rho + P.D);        // per graph: row_ptr [Rcap + 1], row_pdf [Rcap], states [Kcap]
    const uint16_t *rp[2], *rd[2], *rs[2];
    PdfSub ps[2];
    // The first graph's rows of the next frame travel from HBM into registers while the current frame is
    // worked on (when it is a shared graph of float vectors whose rows are 16-byte aligned).
    const PostGraph &G0 = P.g[0];
    const int K0 = G0.pdfs.sub[0].K;
    const bool pre = G0.shared && !G0.f64 && (K0 & 3) == 0 && (G0.ld & 3) == 0 && (((uintptr_t)G0.a | (uintptr_t)G0.b) & 15) == 0 &&
                     n0 < n_end;
    const int Kpre = pre ? min(K0, NT * 4 * U) : 0;   // states covered by the prefetch registers
    float4 pa[U], pb[U];
    auto issue = [&](int n) {
        const float4 *ar = (const float4 *)((const float *)G0.a + ((size_t)b * P.N + n) * G0.ld);
        const float4 *br = (const float4 *)((const float *)G0.b + ((size_t)b * P.N + n) * G0.ld);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int q = u * NT + tid;
            if (q * 4 < Kpre) { pa[u] = ar[q]; pb[u] = br[q]; }
        }
    };
    if (pre) issue(n0);
    if (n0 < n_end) {   // the tables are needed only if the chunk has a real frame
        uint16_t *at = tab;
        for (int gi = 0; gi < P.n_graph; ++gi) {
            const PostGraph &G = P.g[gi];
            ps[gi] = G.pdfs.sub[G.shared ? 0 : b];
            uint16_t *p0 = at, *p1 = p0 + G.Rcap + 1, *p2 = p1 + G.Rcap;
            for (int r = tid; r <= ps[gi].n_rows; r += NT) p0[r] = G.pdfs.row_ptr[ps[gi].ptr0 + r];
            for (int r = tid; r < ps[gi].n_rows; r += NT) p1[r] = G.pdfs.row_pdf[ps[gi].row0 + r];
            for (int k = tid; k < ps[gi].K; k += NT) p2[k] = G.pdfs.states[ps[gi].st0 + k];
            rp[gi] = p0; rd[gi] = p1; rs[gi] = p2;
            at = p0 + ((2 * G.Rcap + 1 + G.Kcap + 1) & ~1);   // next table starts 4-byte aligned
        }
        __syncthreads();
    }

    for (int fi = 0; fi < P.frames_per_block; ++fi) {
        const int n = n0 + fi;
        if (n >= P.N) break;
        float *prow = P.pdf_out ? P.pdf_out + ((size_t)b * P.N + n) * P.D : nullptr;
        if (n >= T) {   // padded frame: zeros
            if (P.accumulate) continue;
            if (prow)
                for (int d = tid; d < P.D; d += NT) prow[d] = 0.0f;
            for (int gi = 0; gi < P.n_graph; ++gi) {
                const PostGraph &G = P.g[gi];
                if (!G.state_post) continue;
                const PdfSub sd = G.pdfs.sub[G.shared ? 0 : b];
                float *srow = G.shared ? G.state_post + ((size_t)b * P.N + n) * sd.K
                                       : G.state_post + (size_t)n * G.Ktot + sd.k0;
                for (int k = tid; k < sd.K; k += NT) srow[k] = 0.0f;
            }
            continue;
        }
        for (int gi = 0; gi < P.n_graph; ++gi) {
            const PostGraph &G = P.g[gi];
            const int K = ps[gi].K;
            const size_t at = G.shared ? ((size_t)b * P.N + n) * G.ld : (size_t)n * G.Ktot + ps[gi].k0;
            const bool covers_all = G.shared != 0;   // a shared graph has one row per pdf
            if (gi == 0 && !covers_all && prow && !P.accumulate)
                for (int d = tid; d < P.D; d += NT) rho[d] = 0.0f;
            float inv;
            if (G.f64) {
                const double mx = frame_logpost<double>((const double *)G.a + at, (const double *)G.b + at, (double)G.in_scale, K,
                                                        stage64, tid);
                inv = frame_finish<double>(mx, K, tb, stage64, red, tid, lane, wave);
            } else if (gi == 0 && pre) {
                float mx = -INFINITY;   // this frame's rows are in the registers
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int q = u * NT + tid;
                    if (q * 4 < Kpre) {
                        float4 t;
                        t.x = (pa[u].x + pb[u].x) * G.in_scale; t.y = (pa[u].y + pb[u].y) * G.in_scale;
                        t.z = (pa[u].z + pb[u].z) * G.in_scale; t.w = (pa[u].w + pb[u].w) * G.in_scale;
                        ((float4 *)tb)[q] = t;
                        mx = tmax(tmax(mx, tmax(t.x, t.y)), tmax(t.z, t.w));
                    }
                }
                if (n + 1 < n_end) issue(n + 1);   // the next frame starts its trip now
                if (K > Kpre)
                    mx = tmax(mx, frame_logpost<float>((const float *)G.a + at + Kpre, (const float *)G.b + at + Kpre,
                                                       G.in_scale, K - Kpre, tb + Kpre, tid));
                inv = frame_finish<float>(mx, K, tb, tb, red, tid, lane, wave);
            } else {
                const float mx = frame_logpost<float>((const float *)G.a + at, (const float *)G.b + at, G.in_scale, K, tb, tid);
                inv = frame_finish<float>(mx, K, tb, tb, red, tid, lane, wave);
            }
            if (G.state_post) {
                float *srow = G.state_post + (G.shared ? ((size_t)b * P.N + n) * K : at);
                for (int k = tid; k < K; k += NT) srow[k] = tb[k] * inv;
            }
            __syncthreads();   // tb complete (and red free again)
            if (prow) {
                const float scale = G.sign * inv;
                const uint16_t *ptr = rp[gi], *pdfid = rd[gi], *st = rs[gi];
                const int n_rows = ps[gi].n_rows;
                // tpr threads share a pdf when there are fewer pdfs than threads (tpr a power of two <= 16);
                // each thread walks two pdfs at once so that two chains of dependent LDS reads overlap
                int tpr = 1;
                while (tpr < 16 && n_rows * tpr * 2 <= NT) tpr *= 2;
                const int rpp = NT / tpr, part = tid & (tpr - 1);
                for (int r0 = tid / tpr; r0 < n_rows; r0 += 2 * rpp) {
                    const int r1 = r0 + rpp;
                    const bool two = r1 < n_rows;
                    int i0 = ptr[r0] + part, i1 = two ? ptr[r1] + part : 0;
                    const int e0 = ptr[r0 + 1], e1 = two ? ptr[r1 + 1] : 0;
                    float acc0 = 0.0f, acc1 = 0.0f;
                    while (i0 < e0 || i1 < e1) {
                        const float v0 = i0 < e0 ? tb[st[i0]] : 0.0f, v1 = i1 < e1 ? tb[st[i1]] : 0.0f;
                        acc0 += v0; acc1 += v1;
                        i0 += tpr; i1 += tpr;
                    }
                    for (int o = tpr >> 1; o >= 1; o >>= 1) {   // fixed order: results do not depend on timing
                        acc0 += __shfl_xor(acc0, o, 64);
                        acc1 += __shfl_xor(acc1, o, 64);
                    }
                    if (part == 0) {
                        if (P.accumulate) {   // straight into the caller's row: a sequence's rows name distinct pdfs
                            prow[pdfid[r0]] += acc0 * scale;
                            if (two) prow[pdfid[r1]] += acc1 * scale;
                        } else {
                            if (gi == 0 && covers_all) rho[pdfid[r0]] = acc0 * scale;
                            else rho[pdfid[r0]] += acc0 * scale;
                            if (two) {
                                if (gi == 0 && covers_all) rho[pdfid[r1]] = acc1 * scale;
                                else rho[pdfid[r1]] += acc1 * scale;
                            }
                        }
                    }
                }
                __syncthreads();
            }
        }
        if (prow && !P.accumulate)
            for (int d = tid; d < P.D; d += NT) prow[d] = rho[d];
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// Gradient of the LF-MMI objective (Eq. 17) for the usual pair of graphs: a shared
// denominator whose vectors are float, packed numerators with at most kGradNumK
// states and pdf rows each (or the denominator's share alone), for calls whose
// recursions also left the running sums of their offsets (PostParams::cum_a, cum_b:
// A_n, B_n with alpha_n = stored row + A_n, beta_n = stored row + B_n, log2 units)
// and log Z.  Same sums in the same order as fb_posterior_kernel, organised for speed:
// grid = (ceil(N / frames_per_block), B), 8 waves, one workgroup barrier per frame.  (Eight, two per SIMD: two
// workgroups then share a compute unit.  With nine - three on one SIMD - the second workgroup was never placed
// beside the first, whatever the occupancy calculation says, and the kernel ran at 3/4 of its present rate.)
// Waves 0-6 work on the denominator: a thread keeps, for the whole block, the
// places of "its" states in pdf order and the state ranges of "its" pdfs in
// registers, the rows of the next frame travel from HBM into registers while the
// current frame is worked on, and the exponentials go to LDS in pdf order, so that a
// pdf's states are neighbours.  The exponentials of a frame are taken of
//   t_k - (log2 Z - A_n - B_n) = log2 of the posterior itself (<= 0, largest >= -log2 K),
// so no maximum over the frame, no reduction of it over the workgroup and no barrier
// behind it are needed (the values are still normalised by their own sum, so a drift
// of the float recursions cancels).  The denominator waves store their pdf posteriors
// straight from the sums (no staging of the row in LDS), adding the numerator's value
// for the pdf, which wave 7 - it works on the numerator of the same frame at the same
// time, with wave-level reductions only - has left in a small list (two buffers, by
// frame parity) before the frame's barrier; the exponentials in pdf order have two
// buffers as well, so nothing of frame n + 1 overwrites what frame n still reads.
// Without the offsets (the pdf posteriors of fb_posteriors: one shared graph, rows of logarithms as fb_alpha and
// fb_beta return them) the frame's largest sum of a forward and a backward entry takes the place of
// log2 Z - A_n - B_n: one more reduction over the workgroup and a second barrier per frame.
// LDS: red [2][16] sums and [2][16] maxima of waves 0-6; tb [2][K0 rounded to 4, + kGradSlack]; nval [2][Rcap] the numerator's pdf
// posteriors by pdf row; en [Kcap] numerator exponentials; nidx [D] 16-bit: pdf -> its row in
// this sequence's numerator + 1, 0 = none; the numerator tables.
// ---------------------------------------------------------------------------
constexpr int kGradMain = 448, kGradThreads = kGradMain + kWave;
constexpr int kGradU = 4;        // 16-byte pieces of a denominator row per thread: 7168 states
constexpr int kGradPdf = 8;      // pdfs per thread: 3584 pdfs
constexpr int kGradNumU = 8;     // numerator states (and pdf rows) per lane: 512
constexpr int kGradNumK = kGradNumU * kWave;
constexpr int kGradAhead = 8;    // states of a pdf whose exponentials are read at once, before any of them is added
constexpr int kGradSlack = 4 + kGradAhead;   // floats behind a buffer of exponentials: reads ahead may pass the last state

// a 16-byte load of data that is read once: it should not push the recursion kernel's arc plan out of L2
__device__ __forceinline__ float4 nt_load4(const float4 *p)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    const f4 v = __builtin_nontemporal_load((const f4 *)p);
    return make_float4(v.x, v.y, v.z, v.w);
}

// four consecutive floats of a row whose pieces need not be 16-byte aligned; have: how many of them exist (the
// others come back as 0 and nothing behind the row is touched)
__device__ __forceinline__ float4 nt_load4_any(const float *p, int have)
{
    typedef float f4u __attribute__((ext_vector_type(4), aligned(4)));
    if (have >= 4) {
        const f4u v = __builtin_nontemporal_load((const f4u *)p);
        return make_float4(v.x, v.y, v.z, v.w);
    }
    float4 r = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (have > 0) r.x = p[0];
    if (have > 1) r.y = p[1];
    if (have > 2) r.z = p[2];
    return r;
}

template <class NT>
__global__ __launch_bounds__(kGradThreads, 4) void fb_grad_kernel(const PostParams P)
{
    extern __shared__ double lds_raw[];
    constexpr int MT = kGradMain, U = kGradU, NU = kGradNumU;
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool den_side = wave < MT / kWave;
    const int b = P.order ? P.order[P.rank0 + blockIdx.y] : blockIdx.y;
    const int T = min(max(P.lengths[b], 0), P.N);
    const int n0 = blockIdx.x * P.frames_per_block;
    const int n_end = min(min(n0 + P.frames_per_block, P.N), T);   // real frames of this chunk: [n0, n_end)
    // one graph, or a second graph whose vectors were not complete when the launch was released (PostParams::fused):
    // the shared graph's share alone (no numerators: wave 7 only keeps the barriers)
    const bool has_num = P.n_graph == 2 && (!P.fused || *P.fused != 0);
    const PostGraph &G0 = P.g[0], &G1 = P.g[1];
    const int K0 = G0.pdfs.sub[0].K, D = P.D;
    const int K0r = ((K0 + 3) & ~3) + kGradSlack;
    const PdfSub ps1 = has_num ? G1.pdfs.sub[b] : PdfSub{};
    const int K1 = ps1.K, R1 = ps1.n_rows;

    float *red = (float *)lds_raw;                       // [2][16] sums, [2][16] maxima
    float *tb = red + 64;                                // [2][K0r]
    float *nval = tb + 2 * K0r;                          // [2][Rcap]
    float *en = nval + 2 * G1.Rcap;                      // [Kcap]
    uint16_t *nidx = (uint16_t *)(en + G1.Kcap);         // [D rounded to 2]
    uint16_t *nptr = nidx + ((D + 1) & ~1);              // numerator tables: row_ptr [Rcap + 1], row_pdf [Rcap], states [Kcap]
    uint16_t *npdf = nptr + G1.Rcap + 1, *nst = npdf + G1.Rcap;

    for (int n = n0 + (n_end > n0 ? n_end - n0 : 0); n < min(n0 + P.frames_per_block, P.N); ++n) {   // padded frames: zeros
        float *prow = P.pdf_out + ((size_t)b * P.N + n) * D;
        for (int d = tid; d < D; d += kGradThreads) prow[d] = 0.0f;
    }
    if (n0 >= n_end) return;

    // which numerator row a pdf has (the same for every frame of the block)
    for (int d = tid; d < D; d += kGradThreads) nidx[d] = 0;
    __syncthreads();
    for (int r = tid; r < R1; r += kGradThreads) nidx[G1.pdfs.row_pdf[ps1.row0 + r]] = (uint16_t)(r + 1);   // (R1 = 0 without numerators)
    // (visible to the denominator waves after the first frame's barrier)

    if (den_side) {
        float4 pa[U], pb[U];          // rows of the frame being prefetched / worked on
        float ca, cb;                 // A_n, B_n of that frame
        uint2 posr[U];                // places (4 x 16 bit) of the thread's states in pdf order
        uint32_t prange[kGradPdf];    // state ranges (begin | end << 16) of the thread's pdfs tid, tid + MT, ...
        const double z2 = P.logz ? P.logz[b] * kLog2e : 0.0;   // log2 Z of the shared graph
        // rows in whole 16-byte pieces (the workspace of an LF-MMI call; the caller's rows when K is a multiple of 4)
        const bool pieces16 = (G0.ld & 3) == 0 && (((uintptr_t)G0.a | (uintptr_t)G0.b) & 15) == 0;
        const bool by_max = !P.cum_a;   // no offsets: the frame's exponentials are taken relative to its largest sum
        // the form of this sequence's rows: the values themselves (what the probability-domain recursion leaves), or logs
        const bool lin_a = G0.fmt_a && G0.fmt_a[b] != 0, lin_b = G0.fmt_b && G0.fmt_b[b] != 0;
        const bool any_lin = lin_a || lin_b;
        const float in_scale0 = G0.in_scale;
        auto as_value = [in_scale0](float v, bool lin) -> double {   // a row entry as a double: itself, or 2^(its log2)
            if (lin) return (double)v;
            const float x = v * in_scale0;
            if (!(x > -1.0e30f)) return 0.0;
            const float fl = floorf(x);
            return ldexp((double)fexp2(x - fl), (int)fl);
        };
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int q = u * MT + tid;
            posr[u] = q * 4 < K0 ? ((const uint2 *)G0.pdfs.pos)[q] : make_uint2(0u, 0u);
        }
        // Few pdfs (the paper's own graphs: 84 pdfs for 3022 states): tpp threads, neighbours in a wave, share a pdf,
        // each with a part of its states; their sums are added in a fixed order.  Otherwise a thread has up to
        // kGradPdf whole pdfs: tid, tid + MT, ...
        int tpp = 1;
        while (tpp < kWave && D * tpp * 2 <= MT) tpp *= 2;
        const int n_mine = tpp > 1 ? 1 : kGradPdf;   // pdfs (or parts of one) of a thread
#pragma unroll
        for (int j = 0; j < kGradPdf; ++j) {
            const int d = tpp > 1 ? tid / tpp : j * MT + tid;
            uint32_t lo = 0, hi = 0;
            if (d < D && j < n_mine) {
                lo = G0.pdfs.row_ptr[d];
                hi = G0.pdfs.row_ptr[d + 1];
                if (tpp > 1) {
                    const uint32_t len = hi - lo, part = (uint32_t)(tid & (tpp - 1));
                    hi = lo + len * (part + 1) / (uint32_t)tpp;
                    lo = lo + len * part / (uint32_t)tpp;
                }
            }
            prange[j] = lo | (hi << 16);
        }
        // the most states any pdf of this wave has: how far the reads ahead below go is the same for all its lanes
        float most = 0.0f;
#pragma unroll
        for (int j = 0; j < kGradPdf; ++j) most = tmax(most, (float)((prange[j] >> 16) - (prange[j] & 0xffffu)));
        const int wcnt = __builtin_amdgcn_readfirstlane((int)wave_max(most));
        // The frames of the block, for one form of the rows: 2 both hold values (every sequence the probability-domain
        // recursion has carried through), 0 both hold logs, 1 one of each (a sequence that fell back in one direction).
        auto frames = [&](auto form_c, auto few_c) {
        constexpr int form = decltype(form_c)::value;
        constexpr bool few = decltype(few_c)::value;   // few pdfs: several threads share one (tpp > 1)
        auto issue = [&](int n) {
            const float *af = (const float *)G0.a + ((size_t)b * P.N + n) * G0.ld;
            const float *bf = (const float *)G0.b + ((size_t)b * P.N + n) * G0.ld;
            const float4 *ar = (const float4 *)af, *br = (const float4 *)bf;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int q = u * MT + tid;
                if (q * 4 < K0) {
                    // (rows that hold values are the workspace's: whole pieces)
                    if (form != 0 || pieces16) { pa[u] = nt_load4(ar + q); pb[u] = nt_load4(br + q); }
                    else { pa[u] = nt_load4_any(af + q * 4, K0 - q * 4); pb[u] = nt_load4_any(bf + q * 4, K0 - q * 4); }
                }
            }
            ca = (form == 0 && by_max) ? 0.0f : P.cum_a[(size_t)b * P.N + n];   // (rows that hold values come with offsets)
            cb = (form == 0 && by_max) ? 0.0f : P.cum_b[(size_t)b * P.N + n];
        };
        issue(n0);
        for (int n = n0; n < n_end; ++n) {
            const int par = (n - n0) & 1;
            float *tbn = tb + par * K0r;
            // (the packed places and ranges stay packed between frames: unpacked once and for all they would not fit
            // the registers)
#pragma unroll
            for (int u = 0; u < U; ++u) asm volatile("" : "+v"(posr[u].x), "+v"(posr[u].y));
#pragma unroll
            for (int j = 0; j < kGradPdf; ++j) asm volatile("" : "+v"(prange[j]));
            // log2 Z - A_n - B_n; a sequence without any path (log Z = -inf) has no posteriors
            double shift_d = z2 - (double)ca - (double)cb;
            if (form == 0 && by_max) {
                // Rows without offsets (normalised logs as fb_alpha / fb_beta return them): the largest sum of the
                // frame takes the place of log2 Z - A_n - B_n, at the price of a second barrier per frame.
                float mx = -INFINITY;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int q = u * MT + tid;
                    if (q * 4 < K0) {
                        mx = tmax(mx, pa[u].x + pb[u].x);
                        if (q * 4 + 1 < K0) mx = tmax(mx, pa[u].y + pb[u].y);
                        if (q * 4 + 2 < K0) mx = tmax(mx, pa[u].z + pb[u].z);
                        if (q * 4 + 3 < K0) mx = tmax(mx, pa[u].w + pb[u].w);
                    }
                }
                mx = wave_max(mx);
                if (lane == 0) red[32 + par * 16 + wave] = mx;
                __syncthreads();
                mx = red[32 + par * 16];
#pragma unroll
                for (int w = 1; w < MT / kWave; ++w) mx = tmax(mx, red[32 + par * 16 + w]);
                shift_d = mx > -INFINITY ? (double)(mx * G0.in_scale) : -INFINITY;
            }
            const bool mass = shift_d > -1.0e300 && shift_d < 1.0e300;
            const float shift = mass ? (float)shift_d : 0.0f;
            // 2^-shift in double, for rows that hold values instead of logs (their range is a float's, times the offsets')
            double pow_shift = 0.0;
            if (form != 0 && mass) {
                const double t = fmin(fmax(-shift_d, -2000.0), 2000.0), ti = floor(t);
                pow_shift = ldexp((double)fexp2((float)(t - ti)), (int)ti);
            }
            float sum = 0.0f;
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int q = u * MT + tid;
                if (q * 4 < K0) {
                    float e[4];
                    if (form == 2) {   // rows that hold the values themselves: the posterior is their product, formed in double
                        e[0] = (float)((double)pa[u].x * (double)pb[u].x * pow_shift);
                        e[1] = (float)((double)pa[u].y * (double)pb[u].y * pow_shift);
                        e[2] = (float)((double)pa[u].z * (double)pb[u].z * pow_shift);
                        e[3] = (float)((double)pa[u].w * (double)pb[u].w * pow_shift);
                    } else if (form == 1) {
                        e[0] = (float)(as_value(pa[u].x, lin_a) * as_value(pb[u].x, lin_b) * pow_shift);
                        e[1] = (float)(as_value(pa[u].y, lin_a) * as_value(pb[u].y, lin_b) * pow_shift);
                        e[2] = (float)(as_value(pa[u].z, lin_a) * as_value(pb[u].z, lin_b) * pow_shift);
                        e[3] = (float)(as_value(pa[u].w, lin_a) * as_value(pb[u].w, lin_b) * pow_shift);
                    } else {
                        e[0] = fexp2((pa[u].x + pb[u].x) * G0.in_scale - shift); e[1] = fexp2((pa[u].y + pb[u].y) * G0.in_scale - shift);
                        e[2] = fexp2((pa[u].z + pb[u].z) * G0.in_scale - shift); e[3] = fexp2((pa[u].w + pb[u].w) * G0.in_scale - shift);
                    }
                    if (q * 4 + 3 >= K0) {   // the row's last piece when K0 is not a multiple of 4: padding counts as zero-bar
                        if (q * 4 + 1 >= K0) e[1] = 0.0f;
                        if (q * 4 + 2 >= K0) e[2] = 0.0f;
                        e[3] = 0.0f;
                    }
                    if (!mass) e[0] = e[1] = e[2] = e[3] = 0.0f;
                    sum += (e[0] + e[1]) + (e[2] + e[3]);
                    tbn[posr[u].x & 0xffffu] = e[0]; tbn[posr[u].x >> 16] = e[1];
                    tbn[posr[u].y & 0xffffu] = e[2]; tbn[posr[u].y >> 16] = e[3];
                }
                __builtin_amdgcn_sched_barrier(0);   // one piece at a time: the doubles of all at once would not fit the registers
            }
            if (n + 1 < n_end) issue(n + 1);   // the next frame starts its trip now
            sum = wave_sum(sum);
            if (lane == 0) red[par * 16 + wave] = sum;
            __syncthreads();                       // the frame's only barrier
            sum = red[par * 16];
#pragma unroll
            for (int w = 1; w < MT / kWave; ++w) sum += red[par * 16 + w];
            const float scale = sum > 0.0f ? G0.sign / sum : 0.0f;
            float *prow = P.pdf_out + ((size_t)b * P.N + n) * D;
            const float *nv = nval + par * G1.Rcap;
            // A pdf's exponentials are neighbours in the buffer.  The first kGradAhead of each of two pdfs are read
            // at once (as far as the wave's longest pdf goes; what lies behind a pdf's own states is read and not
            // used), so that a thread waits for LDS once per two pdfs and not once per state; they are added in
            // ascending order of states as before, and what a pdf has beyond them in a loop of its own.
            constexpr int H = 2;
            static_assert(kGradPdf % H == 0, "pdfs per thread come in groups");
#pragma unroll
            for (int h = 0; h < (few ? 1 : kGradPdf); h += H) {
                float t[H][kGradAhead];
                uint32_t r[H];
#pragma unroll
                for (int jj = 0; jj < H; ++jj) {
                    const float *seg = tbn + (prange[h + jj] & 0xffffu);
#pragma unroll
                    for (int i = 0; i < kGradAhead; i += 2)
                        if (wcnt > i) { t[jj][i] = seg[i]; t[jj][i + 1] = seg[i + 1]; }
                    r[jj] = nidx[min(few ? tid / tpp : (h + jj) * MT + tid, D - 1)];
                }
                float nvv[H];
#pragma unroll
                for (int jj = 0; jj < H; ++jj) nvv[jj] = nv[r[jj] ? r[jj] - 1 : 0];   // (no numerators: never used)
#pragma unroll
                for (int jj = 0; jj < H; ++jj) {
                    const int d = few ? tid / tpp : (h + jj) * MT + tid;
                    const int begin = (int)(prange[h + jj] & 0xffffu), end = (int)(prange[h + jj] >> 16);
                    float acc = 0.0f;
#pragma unroll
                    for (int i = 0; i < kGradAhead; ++i)
                        if (wcnt > i) acc += begin + i < end ? t[jj][i] : 0.0f;
                    if (wcnt > kGradAhead)
                        for (int i = begin + kGradAhead; i < end; ++i) acc += tbn[i];
                    if (few)
                        for (int o = 1; o < tpp; o <<= 1) acc += __shfl_xor(acc, o, kWave);   // the parts of a pdf, in a fixed order
                    // (a product and a sum, each rounded: the bits a launch of the denominator's share followed by one
                    // that adds the numerators' gives, whichever of the two ways a call takes)
                    float v = acc * scale;
                    asm volatile("" : "+v"(v));   // (kept a product of its own: not merged with the sum into one rounding)
                    if (r[jj]) v += nvv[jj];
                    if (few ? (d < D && (tid & (tpp - 1)) == 0 && jj == 0) : d < D) __builtin_nontemporal_store(v, prow + d);
                }
            }
        }
        };
        const std::true_type yes;
        const std::false_type no;
        if (tpp > 1) {
            if (lin_a && lin_b) frames(std::integral_constant<int, 2>(), yes);
            else if (any_lin) frames(std::integral_constant<int, 1>(), yes);
            else frames(std::integral_constant<int, 0>(), yes);
        } else {
            if (lin_a && lin_b) frames(std::integral_constant<int, 2>(), no);
            else if (any_lin) frames(std::integral_constant<int, 1>(), no);
            else frames(std::integral_constant<int, 0>(), no);
        }
    } else {
        NT qa[NU], qb[NU];            // rows of the frame being prefetched / worked on
        auto issue = [&](int n) {
            const NT *ar = (const NT *)G1.a + (size_t)n * G1.Ktot + ps1.k0, *br = (const NT *)G1.b + (size_t)n * G1.Ktot + ps1.k0;
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int k = u * kWave + lane;
                if (k < K1) { qa[u] = ar[k]; qb[u] = br[k]; }
            }
        };
        if (!has_num) {
            const bool two = !P.cum_a && !(G0.fmt_a && G0.fmt_a[b] != 0) && !(G0.fmt_b && G0.fmt_b[b] != 0);   // as the other waves decide
            for (int n = n0; n < n_end; ++n) {
                if (two) __syncthreads();
                __syncthreads();
            }
            return;
        }
        issue(n0);
        for (int r = lane; r <= R1; r += kWave) nptr[r] = G1.pdfs.row_ptr[ps1.ptr0 + r];
        for (int k = lane; k < K1; k += kWave) nst[k] = G1.pdfs.states[ps1.st0 + k];
        for (int n = n0; n < n_end; ++n) {
            const int par = (n - n0) & 1;
            NT t[NU];
            NT mx = (NT)(-INFINITY);
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int k = u * kWave + lane;
                if (k < K1) {
                    t[u] = (qa[u] + qb[u]) * (NT)G1.in_scale;
                    mx = tmax(mx, t[u]);
                }
            }
            if (n + 1 < n_end) issue(n + 1);
            mx = wave_max(mx);
            float sum = 0.0f;
            const bool mass = mx != (NT)(-INFINITY);
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the previous frame's reads of en come first
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int k = u * kWave + lane;
                if (k < K1) {
                    const float e = mass ? fexp2((float)(t[u] - mx)) : 0.0f;
                    en[k] = e;
                    sum += e;
                }
            }
            sum = wave_sum(sum);
            const float scale = sum > 0.0f ? G1.sign / sum : 0.0f;
            __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");   // the wave's writes of en (and of its tables) before its reads
            float *nv = nval + par * G1.Rcap;
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int r = u * kWave + lane;
                if (r < R1) {
                    float acc = 0.0f;
                    for (int i = nptr[r]; i < nptr[r + 1]; ++i) acc += en[nst[i]];
                    nv[r] = acc * scale;
                }
            }
            __syncthreads();                       // the frame's only barrier: the denominator waves may read nv
        }
    }
}

// The pdf posteriors of small packed graphs (at most kGradNumK states and pdf rows each; the numerators of an
// LF-MMI call) added, with the graph's sign, to rows that already hold another graph's share (PostParams::accumulate).
// grid = (ceil(N / frames_per_block), B), one wave per workgroup: the wave walks its frames as the last wave of
// fb_grad_kernel does (same arithmetic, same order), with the rows of the next frame on their way while it works,
// and adds straight into the caller's rows: a sequence's pdf rows name distinct pdfs, padded frames are left alone.
template <class NT>
__global__ __launch_bounds__(kWave) void fb_num_add_kernel(const PostParams P)
{
    extern __shared__ double lds_raw[];
    constexpr int NU = kGradNumU;
    const int lane = threadIdx.x;
    const int b = P.order ? P.order[P.rank0 + blockIdx.y] : blockIdx.y;
    const int T = min(max(P.lengths[b], 0), P.N);
    const int n0 = blockIdx.x * P.frames_per_block;
    const int n_end = min(n0 + P.frames_per_block, T);   // real frames of this chunk: [n0, n_end)
    if (n0 >= n_end) return;
    if (P.fused && *P.fused != 0) return;   // the launch before this one has added this graph's share already
    const PostGraph &G1 = P.g[0];
    const PdfSub ps1 = G1.pdfs.sub[b];
    const int K1 = ps1.K, R1 = ps1.n_rows;
    float *en = (float *)lds_raw;                        // [Kcap] exp(log posterior - max)
    uint16_t *nptr = (uint16_t *)(en + G1.Kcap);         // row_ptr [Rcap + 1], row_pdf [Rcap], states [Kcap]
    uint16_t *npdf = nptr + G1.Rcap + 1, *nst = npdf + G1.Rcap;
    NT qa[NU], qb[NU];
    auto issue = [&](int n) {
        const NT *ar = (const NT *)G1.a + (size_t)n * G1.Ktot + ps1.k0, *br = (const NT *)G1.b + (size_t)n * G1.Ktot + ps1.k0;
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int k = u * kWave + lane;
            if (k < K1) { qa[u] = ar[k]; qb[u] = br[k]; }
        }
    };
    issue(n0);
    for (int r = lane; r <= R1; r += kWave) nptr[r] = G1.pdfs.row_ptr[ps1.ptr0 + r];
    for (int r = lane; r < R1; r += kWave) npdf[r] = G1.pdfs.row_pdf[ps1.row0 + r];
    for (int k = lane; k < K1; k += kWave) nst[k] = G1.pdfs.states[ps1.st0 + k];
    for (int n = n0; n < n_end; ++n) {
        NT t[NU];
        NT mx = (NT)(-INFINITY);
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int k = u * kWave + lane;
            if (k < K1) {
                t[u] = (qa[u] + qb[u]) * (NT)G1.in_scale;
                mx = tmax(mx, t[u]);
            }
        }
        if (n + 1 < n_end) issue(n + 1);
        mx = wave_max(mx);
        float sum = 0.0f;
        const bool mass = mx != (NT)(-INFINITY);
        __syncthreads();   // (one wave: orders the previous frame's reads of en before these writes)
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int k = u * kWave + lane;
            if (k < K1) {
                const float e = mass ? fexp2((float)(t[u] - mx)) : 0.0f;
                en[k] = e;
                sum += e;
            }
        }
        sum = wave_sum(sum);
        const float scale = sum > 0.0f ? G1.sign / sum : 0.0f;
        __syncthreads();   // the writes of en (and, in the first frame, of the tables) before the reads below
        float *prow = P.pdf_out + ((size_t)b * P.N + n) * P.D;
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const int r = u * kWave + lane;
            if (r < R1) {
                float acc = 0.0f;
                for (int i = nptr[r]; i < nptr[r + 1]; ++i) acc += en[nst[i]];
                float share = acc * scale;
                asm volatile("" : "+v"(share));   // (rounded as the gradient kernel's last wave rounds it, then added)
                prow[npdf[r]] += share;
            }
        }
    }
}

// order[rank] = b: the sequences by length, longest first (equal lengths by index).  One thread per sequence
// counts the sequences that go before its own.
__global__ __launch_bounds__(256) void fb_order_kernel(const int32_t *lengths, int32_t B, int32_t N, int32_t *order, uint32_t *done)
{
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (done && b <= kDoneStarted) done[b] = 0u;   // the progress counters of the call start at zero
    if (b >= B) return;
    const int lb = min(max(lengths[b], 0), N);
    int rank = 0;
    for (int j = 0; j < B; ++j) {
        const int lj = min(max(lengths[j], 0), N);
        rank += (lj > lb || (lj == lb && j < b)) ? 1 : 0;
    }
    order[rank] = b;
}

// loss = sum_b (log Z_num[b] - log Z_den[b]) over the sequences that have frames (Eq. 16),
// summed in double in a fixed order.
__global__ __launch_bounds__(256) void fb_loss_kernel(const double *zn, const double *zd, const int32_t *lengths, int32_t B,
                                                      double *loss)
{
    __shared__ double acc[256];
    double a = 0.0;
    for (int b = threadIdx.x; b < B; b += 256)
        if (lengths[b] > 0) a += zn[b] - zd[b];
    acc[threadIdx.x] = a;
    __syncthreads();
    for (int s = 128; s >= 1; s >>= 1) {
        if ((int)threadIdx.x < s) acc[threadIdx.x] += acc[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) *loss = acc[0];
}

// Best path from the back-pointers: one thread per sequence walks from the best end state to frame 0.
// Indices are those of the state buffer (a state, or Kcap + slot for a clone of a very long row); a clone
// is reported as the state it belongs to.
// One workgroup per sequence.  A path is a chain of dependent reads (the back-pointer of frame n names the row
// entry to read at frame n - 1), each a trip to HBM if taken one by one; so the workgroup copies the sequence's
// back-pointer rows of kBtFrames frames at a time into LDS (whole rows: which entry is needed is only known once the
// chain gets there), the next block travelling while one thread walks the frames of this one there.
constexpr int kBtThreads = 256, kBtFrames = 8;

__global__ __launch_bounds__(kBtThreads) void fb_backtrace_kernel(const BacktraceParams P)
{
    extern __shared__ uint16_t bt_rows[];   // [frames][W]: the 16-byte pieces that hold the states' columns, then the clone slots'
    const int b = blockIdx.x, tid = threadIdx.x;
    const SubDesc sd = P.sched.sub[P.shared ? 0 : b];
    const CloneDesc *cdesc = P.sched.clones + sd.clone0;
    const int T = min(max(P.lengths[b], 0), P.N);
    int32_t *prow = P.path + (size_t)b * P.N;
    for (int n = T + tid; n < P.N; n += kBtThreads) prow[n] = -1;
    if (T == 0) return;
    const int K = sd.K, F = P.frames;
    // where the sequence's columns lie in a row of back-pointers, and the 16-byte pieces of the row that hold them
    // (rows are a multiple of 8 entries long and start on 16-byte boundaries)
    const int64_t col_states = P.shared ? 0 : sd.k0;
    const int64_t col_clones = P.shared ? (int64_t)K : (int64_t)P.Ktot + (int64_t)b * P.Ccap;
    const int64_t ps0 = col_states >> 3, ps1 = (col_states + K + 7) >> 3;
    const int64_t pc0 = col_clones >> 3, pc1 = (col_clones + P.Ccap + 7) >> 3;
    const int ns = (int)(ps1 - ps0), nc = P.Ccap > 0 ? (int)(pc1 - pc0) : 0;   // pieces
    const int W = (ns + nc) * 8;
    const int at_states = (int)(col_states - ps0 * 8), at_clones = ns * 8 + (int)(col_clones - pc0 * 8);
    const int lane = tid & (kWave - 1), wave = tid >> 6;
    int s = P.last[b];   // index in the kernel's index space: a state, or Kcap + a clone slot (thread 0 follows it)
    if (s < 0) {
        for (int n = tid; n < T; n += kBtThreads) prow[n] = -1;
        return;
    }
    auto state_of = [&](int idx) {
        if (idx < P.Kcap) return idx;
        const int slot = idx - P.Kcap;
        int state = 0;
        for (int j = 0; j < sd.n_cdesc; ++j)
            if (slot >= cdesc[j].first && slot < cdesc[j].first + cdesc[j].count) state = cdesc[j].state;
        return state;
    };
    // frames T-1 .. 1 take their predecessor from their own row; blocks of F rows, highest frame first, in two
    // buffers: the next block is on its way from global memory while thread 0 walks this one
    auto issue = [&](int hi, int buf) {   // rows hi, hi - 1, ..., straight into LDS, 16 bytes per lane, nothing waits in between
        const int cnt = min(F, hi);
        for (int f = 0; f < cnt; ++f) {
            const uint4 *row = (const uint4 *)(P.bp + (P.shared ? ((size_t)b * P.N + (hi - f)) : (size_t)(hi - f)) * P.bp_ld);
            uint4 *dst = (uint4 *)(bt_rows + ((size_t)buf * F + f) * W);
            for (int i0 = wave * kWave; i0 < ns; i0 += kBtThreads)
                if (i0 + lane < ns)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(row + ps0 + i0 + lane),
                                                     (__attribute__((address_space(3))) void *)(dst + i0), 16, 0, 0);
            for (int i0 = wave * kWave; i0 < nc; i0 += kBtThreads)
                if (i0 + lane < nc)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(row + pc0 + i0 + lane),
                                                     (__attribute__((address_space(3))) void *)(dst + ns + i0), 16, 0, 0);
        }
    };
    if (T > 1) issue(T - 1, 0);
    int buf = 0;
    for (int hi = T - 1; hi >= 1; hi -= F, buf ^= 1) {
        const int cnt = min(F, hi);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();   // this block is in LDS; thread 0 has left the other buffer
        if (hi - F >= 1) issue(hi - F, buf ^ 1);
        if (tid == 0) {
            for (int f = 0; f < cnt; ++f) {
                prow[hi - f] = sd.k0 + state_of(s);
                s = bt_rows[((size_t)buf * F + f) * W + (s < P.Kcap ? at_states + s : at_clones + (s - P.Kcap))];
            }
        }
    }
    if (tid == 0) prow[0] = sd.k0 + state_of(s);
}


// ---------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------
static int check_launch(const char *what)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(FB_EHIP, std::string(what) + ": " + hipGetErrorString(e));
    return FB_OK;
}

template <class Kern>
static int launch_rec(Kern kern, int nw, const RecParams &p, size_t lds_bytes, void *stream)
{
    if (lds_bytes > 64 * 1024) {
        const hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return fail(FB_EHIP, std::string("hipFuncSetAttribute(LDS size): ") + hipGetErrorString(e));
    }
    const int32_t n_seq = p.order ? p.n_launch : p.B;
    hipLaunchKernelGGL(kern, dim3((unsigned)(n_seq * p.n_dir)), dim3(nw * kWave), lds_bytes, (hipStream_t)stream, p);
    return check_launch("recursion kernel launch");
}

bool recursion_fixed_available()
{
    // the fixed-buffer instantiation addresses LDS from 0: usable only while the kernel has no static LDS in front
    // of its dynamic array (a property of the build, looked up once)
    static const bool ok = [] {
        hipFuncAttributes attr{};
        hipFuncAttributes attr_lin{};
        hipFuncAttributes attr_prob{};
        const hipError_t e = hipFuncGetAttributes(&attr, (const void *)fb_recursion_kernel<kNWShared, float, false, kXsFixed>);
        const hipError_t e_lin =
            hipFuncGetAttributes(&attr_lin, (const void *)fb_recursion_kernel<kNWShared, float, false, kXsFixed, true>);
        const hipError_t e_prob = hipFuncGetAttributes(&attr_prob, (const void *)fb_linear_kernel);
        return e == hipSuccess && attr.sharedSizeBytes == 0 && e_lin == hipSuccess && attr_lin.sharedSizeBytes == 0 &&
               e_prob == hipSuccess && attr_prob.sharedSizeBytes == 0;
    }();
    return ok;
}

int launch_recursion(int nw, bool f64, bool tropical, const RecParams &p, size_t lds_bytes, void *stream)
{
    if (p.xs_fixed) {   // fixed-length state buffers: large graphs with float vectors only
        if (p.xs_fixed != kXsFixed || nw != kNWShared || f64 || tropical) return fail(FB_EHIP, "internal error: fixed-buffer launch");
        if (p.linear_p) {
            if (!p.shared || p.linear_w) return fail(FB_EHIP, "internal error: probability-domain launch");
            for (int i = 0; i < p.n_dir; ++i) {
                if (!p.dir[i].prob.units) return fail(FB_EHIP, "internal error: probability-domain launch without its plan");
                lds_bytes = std::max(lds_bytes, probability_lds_bytes(p.D, p.dir[i].backward != 0 || (p.dir[i].out && !p.dir[i].out_linear)));
            }
            if (lds_bytes > kLdsBytes) return fail(FB_EHIP, "internal error: probability-domain launch beyond the on-chip memory");
            return launch_rec(fb_linear_kernel, nw, p, lds_bytes, stream);
        }
        if (p.linear_w) return launch_rec(fb_recursion_kernel<kNWShared, float, false, kXsFixed, true>, nw, p, lds_bytes, stream);
        return launch_rec(fb_recursion_kernel<kNWShared, float, false, kXsFixed>, nw, p, lds_bytes, stream);
    }
    if (p.linear_w) return fail(FB_EHIP, "internal error: linear weights without fixed buffers");
    if (tropical) {
        if (nw == kNWShared)
            return f64 ? launch_rec(fb_recursion_kernel<kNWShared, double, true, 0>, nw, p, lds_bytes, stream)
                       : launch_rec(fb_recursion_kernel<kNWShared, float, true, 0>, nw, p, lds_bytes, stream);
        return f64 ? launch_rec(fb_recursion_kernel<kNWSmall, double, true, 0>, nw, p, lds_bytes, stream)
                   : launch_rec(fb_recursion_kernel<kNWSmall, float, true, 0>, nw, p, lds_bytes, stream);
    }
    if (nw == kNWShared)
        return f64 ? launch_rec(fb_recursion_kernel<kNWShared, double, false, 0>, nw, p, lds_bytes, stream)
                   : launch_rec(fb_recursion_kernel<kNWShared, float, false, 0>, nw, p, lds_bytes, stream);
    return f64 ? launch_rec(fb_recursion_kernel<kNWSmall, double, false, 0>, nw, p, lds_bytes, stream)
               : launch_rec(fb_recursion_kernel<kNWSmall, float, false, 0>, nw, p, lds_bytes, stream);
}

size_t probability_lds_bytes(int32_t D, bool staged)
{
    return (size_t)kXbStride + ((size_t)kXsFixed * (staged ? 3 : 1) + 64 + 3 * (((size_t)D + 1 + 3) & ~(size_t)3)) * 4;
}

unsigned int linear_restarts()
{
    unsigned int n = 0;
    if (hipMemcpyFromSymbol(&n, HIP_SYMBOL(g_linear_restarts), sizeof(n)) != hipSuccess) return 0;
    return n;
}

int launch_backtrace(const BacktraceParams &p, void *stream)
{
    // rows of the sequence with the most columns: its states and the clone slots
    BacktraceParams q = p;
    if ((p.bp_ld & 7) != 0 || ((uintptr_t)p.bp & 15) != 0) return fail(FB_EHIP, "internal error: back-pointer rows are not in 16-byte pieces");
    const size_t row_bytes = ((size_t)p.Kcap + (size_t)p.Ccap + 32) * sizeof(uint16_t);   // both spans rounded out to whole pieces
    q.frames = (int32_t)std::max<size_t>(1, std::min<size_t>(kBtFrames, (kLdsBytes - kLdsReserve) / (2 * std::max<size_t>(row_bytes, 1))));   // two buffers
    const size_t lds_bytes = 2 * (size_t)q.frames * row_bytes;
    if (lds_bytes > kLdsBytes) return fail(FB_EUNSUPPORTED, "backtrace: a row of back-pointers exceeds the on-chip memory");
    if (lds_bytes > 64 * 1024) {
        const hipError_t e = hipFuncSetAttribute((const void *)fb_backtrace_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return fail(FB_EHIP, std::string("hipFuncSetAttribute(LDS size): ") + hipGetErrorString(e));
    }
    hipLaunchKernelGGL(fb_backtrace_kernel, dim3((unsigned)p.B), dim3(kBtThreads), lds_bytes, (hipStream_t)stream, q);
    return check_launch("backtrace kernel launch");
}

int launch_posteriors(const PostParams &p, size_t lds_bytes, void *stream)
{
    const dim3 grid((unsigned)((p.N + p.frames_per_block - 1) / p.frames_per_block), (unsigned)(p.order ? p.n_launch : p.B));
    if (lds_bytes > 64 * 1024) {
        const hipError_t e =
            hipFuncSetAttribute((const void *)fb_posterior_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return fail(FB_EHIP, std::string("hipFuncSetAttribute(LDS size): ") + hipGetErrorString(e));
    }
    hipLaunchKernelGGL(fb_posterior_kernel, grid, dim3(kPostThreads), lds_bytes, (hipStream_t)stream, p);
    return check_launch("posterior kernel launch");
}

bool gradient_kernel_applies(const PostParams &p)
{
    if (!p.pdf_out || p.accumulate) return false;
    const bool offsets = p.cum_a && p.cum_b && p.logz;
    if (p.n_graph == 1) {   // the shared graph's share alone: no numerators
        const PostGraph &d = p.g[0];
        // without the offsets of the rows only rows of logarithms (no format flags), relative to each frame's maximum
        if (!offsets && (p.cum_a || p.cum_b || p.logz || d.fmt_a || d.fmt_b)) return false;
        // (rows that are not in whole 16-byte pieces are read piece by piece and need no padding)
        const bool pieces16 = (d.ld & 3) == 0 && d.ld >= ((d.Kcap + 3) & ~3) && (((uintptr_t)d.a | (uintptr_t)d.b) & 15) == 0;
        const bool any_rows = d.ld >= d.Kcap && (((uintptr_t)d.a | (uintptr_t)d.b) & 3) == 0;
        return d.shared && !d.f64 && !d.state_post && d.pdfs.pos && (pieces16 || any_rows) &&
               d.Kcap <= kGradMain * 4 * kGradU && p.D <= kGradMain * kGradPdf;
    }
    if (p.n_graph != 2 || !offsets) return false;
    const PostGraph &d = p.g[0], &n = p.g[1];
    return d.shared && !d.f64 && !d.state_post && d.pdfs.pos && (d.ld & 3) == 0 && d.ld >= ((d.Kcap + 3) & ~3) &&
           d.Kcap <= kGradMain * 4 * kGradU &&
           (((uintptr_t)d.a | (uintptr_t)d.b) & 15) == 0 && p.D <= kGradMain * kGradPdf && !n.shared && !n.state_post &&
           n.Kcap <= kGradNumK && n.Rcap <= kGradNumK;
}

size_t gradient_lds_bytes(const PostParams &p)
{
    const PostGraph &d = p.g[0], &n = p.g[1];
    const size_t nR = p.n_graph == 2 ? (size_t)n.Rcap : 0, nK = p.n_graph == 2 ? (size_t)n.Kcap : 0;   // one graph: no numerator tables
    return 256 + (2 * ((size_t)((d.Kcap + 3) & ~3) + kGradSlack) + 2 * nR + nK) * 4 + ((size_t)((p.D + 1) & ~1) + nR * 2 + 1 + nK + 3) / 2 * 4;
}

int launch_gradient(const PostParams &p, size_t lds_bytes, void *stream)
{
    const dim3 grid((unsigned)((p.N + p.frames_per_block - 1) / p.frames_per_block), (unsigned)(p.order ? p.n_launch : p.B));
    auto kern = p.n_graph == 2 && p.g[1].f64 ? fb_grad_kernel<double> : fb_grad_kernel<float>;
    if (lds_bytes > 64 * 1024) {
        const hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes);
        if (e != hipSuccess) return fail(FB_EHIP, std::string("hipFuncSetAttribute(LDS size): ") + hipGetErrorString(e));
    }
    hipLaunchKernelGGL(kern, grid, dim3(kGradThreads), lds_bytes, (hipStream_t)stream, p);
    return check_launch("gradient kernel launch");
}

bool num_add_kernel_applies(const PostParams &p)
{
    if (p.n_graph != 1 || !p.accumulate || !p.pdf_out) return false;
    const PostGraph &n = p.g[0];
    return !n.shared && !n.state_post && n.Kcap <= kGradNumK && n.Rcap <= kGradNumK;
}

int launch_num_add(const PostParams &p, void *stream)
{
    const PostGraph &n = p.g[0];
    const size_t lds_bytes = (size_t)n.Kcap * 4 + ((size_t)n.Rcap * 2 + 1 + (size_t)n.Kcap + 3) / 2 * 4;
    const dim3 grid((unsigned)((p.N + p.frames_per_block - 1) / p.frames_per_block), (unsigned)(p.order ? p.n_launch : p.B));
    auto kern = n.f64 ? fb_num_add_kernel<double> : fb_num_add_kernel<float>;
    hipLaunchKernelGGL(kern, grid, dim3(kWave), lds_bytes, (hipStream_t)stream, p);
    return check_launch("numerator kernel launch");
}

// Does nothing: a launch whose only effect is that what follows it on its stream starts one launch latency later.
__global__ __launch_bounds__(64) void fb_delay_kernel() {}

// *flag = whether the counter has reached `need` (a progress counter of a launch that may still be running)
__global__ __launch_bounds__(64) void fb_decide_kernel(const uint32_t *count, uint32_t need, int32_t *flag)
{
    if (threadIdx.x == 0) *flag = *(const volatile uint32_t *)count >= need ? 1 : 0;
}

__global__ __launch_bounds__(64) void fb_mark_kernel(uint32_t *word)
{
    if (threadIdx.x == 0) *word = 1u;
}

int launch_mark(uint32_t *word, void *stream)
{
    hipLaunchKernelGGL(fb_mark_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, word);
    return check_launch("mark kernel launch");
}

int launch_decide(const uint32_t *count, uint32_t need, int32_t *flag, void *stream)
{
    hipLaunchKernelGGL(fb_decide_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, count, need, flag);
    return check_launch("decide kernel launch");
}

int launch_delay(void *stream)
{
    hipLaunchKernelGGL(fb_delay_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream);
    return check_launch("delay kernel launch");
}

int launch_order(const int32_t *lengths, int32_t B, int32_t N, int32_t *order, uint32_t *done, void *stream)
{
    hipLaunchKernelGGL(fb_order_kernel, dim3((unsigned)((B + 255) / 256)), dim3(256), 0, (hipStream_t)stream, lengths, B, N, order, done);
    return check_launch("order kernel launch");
}

int launch_loss(const double *zn, const double *zd, const int32_t *lengths, int32_t B, double *loss, void *stream)
{
    hipLaunchKernelGGL(fb_loss_kernel, dim3(1), dim3(256), 0, (hipStream_t)stream, zn, zd, lengths, B, loss);
    return check_launch("loss kernel launch");
}

}  // namespace fb
