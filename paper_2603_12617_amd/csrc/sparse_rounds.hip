// Sparse rounds of the base learners (Sec. 3.1 update inside the ensemble of
// Sec. 3.3) for a high-dimensional iterate that lives in HBM.
//
// A round with nnz non-zero features touches nnz coordinates of every
// learner: the gradient step changes only those, and the projection onto the
// ball is a rescaling, carried by a per-learner scalar (w = sigma * v), so a
// round never sweeps the d coordinates.  The norm needed by the projection
// follows from scalars of the round,
//     ||v - b x_t||^2 = ||v||^2 - 2 b <v, x_t> + b^2 ||x_t||^2,
// carried in float64.
//
// Layout.  The round stream is shared by all runs, so every learner of every
// run touches the SAME coordinates in a round.  V is stored coordinate-major
// with the R*K learners interleaved, V[j][q], q = r*K + i: a lane is a learner,
// one coordinate of the learners of a workgroup is one contiguous row segment
// (256 bytes for 64 learners; rows are padded to an odd number of 128-byte
// lines, see oco_create), every gather and scatter is coalesced and all
// the per-learner scalar work (slope, step, norm, projection) runs
// lane-parallel with no reduction.  A workgroup owns 64, 32, 16, 8 or 4 learners:
// few learners per workgroup spread a small problem over more compute units,
// and a memory instruction then covers several rows at once.
//
// Taking memory out of the chain.  The path is a dependent chain of T rounds
// per learner; a round that gathers from and scatters to HBM costs two memory
// round trips (on gfx9 loads and stores of one wavefront share a counter and
// return out of order, so every gather has to drain the previous scatters).
// In v-space the step is linear, v_t = v_s - sum_{s<=r<t} b_r x_r, hence inside
// a window of 64 rounds
//     <v_t, x_t> = <v_window_start, x_t> - sum_{r<t in window} b_r <x_r, x_t>.
// Per window the kernel therefore has three pieces of work:
//   A  q0_t = <v_start, x_t> for the 64 rounds (bulk gathers);
//   B  one wavefront: the 64 dependent rounds on scalars and LDS only
//      (prediction, slope, step size b_t, norm, projection); the Gram terms
//      <x_r, x_t> come from a pre-pass over the round stream and are almost
//      all zero (two sparse rows rarely share a column); predictions go to LDS;
//   C  V[col] += -b_t x_t[col], the entries split over wavefronts by column so
//      that the updates of one address are issued by one wavefront in round
//      order (bitwise reproducible): no-return float atomics, or, with four
//      learners per workgroup, a plain read-modify-write of the 16 bytes of a
//      row by one lane where the column occurs once in the window; and the
//      window's predictions to Z.
// B is the critical path.  Where the LDS has room for the buffers of three
// windows, A of the next window and C of the previous one run beside B of the
// current one (the kernel below says how); otherwise A, B, C of a window
// follow one another and only the staging of the next window runs beside B.
//
// The comparator's predictions <u_t, x_t> do not depend on the learners and
// are taken by a separate, fully parallel kernel (one thread per run-round).
//
// On the boundary of the ball sigma shrinks geometrically (every projection
// multiplies it by a factor < 1) and v grows, so sigma has to be folded back
// into v now and then: V[:, q] *= sigma_q, ||v||^2 *= sigma_q^2, sigma_q = 1.
// The rounds are launched in segments that end at every 4096th round of the
// horizon; after each segment a grid-wide kernel folds the 64-learner column
// groups whose smallest sigma has dropped below 2^-64 (a streaming pass at HBM
// speed, and a no-op otherwise).  Should a sigma fall below 2^-100 inside a
// segment (steps larger than the ball: sigma then shrinks by a constant factor
// every round), the chain stops after that round and the workgroup folds its
// own columns: all wavefronts apply the window's steps so far, scale the
// columns, measure ||v||^2 exactly (fixed order) and gather the remaining
// rounds' <v, x_t> afresh; then the chain goes on.  Windows are
// aligned to multiples of 64 rounds of the horizon and all fold decisions
// depend on the state and the absolute round index only.
//
// The optimistic two-step update (Eq. (3)) only adds scalars to phase B: the
// played iterate's prediction follows from <w^_t, x_t>, <w^_t, x_{t-1}>,
// <x_{t-1}, x_t> and ||x_{t-1}||^2, so V holds the intermediate model and the
// memory phases are unchanged.
#include "oco_internal.h"

#include <type_traits>
#include <stddef.h>
#include <stdlib.h>
#include "../../include/oco.h"

#include <hip/amd_detail/amd_hip_unsafe_atomics.h>

namespace oco {
namespace {

template <int LOSS> __device__ __forceinline__ float slope(float z, float y)
{
    if (LOSS == 0) return 1.0f;
    if (LOSS == 1) return 2.0f * (z - y);
    return -y * __builtin_amdgcn_rcpf(1.0f + __expf(y * z));
}

// V is updated by float atomics, which execute in L2, or by plain stores, which write through to it: every
// read of V in the window kernel goes to L2 as well, past the compute unit's own cache.  (Plain cached loads with
// that cache dropped once per window measured slower: 23.7 against 20.6 ms on the largest sparse workload.)
__device__ __forceinline__ float ldv(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}
typedef float f4 __attribute__((ext_vector_type(4)));
// 16 bytes of a row of V (four neighbouring learners) by one lane, the same kind of load.  The compiler knows
// nothing of a load inside an asm statement: the caller keeps the result's registers reserved until the load has
// returned, by naming them in the s_waitcnt statement it waits with (wait_ldv4).
__device__ __forceinline__ f4 ldv4(const float *p)
{
    f4 r;
    asm volatile("global_load_dwordx4 %0, %1, off sc0" : "=v"(r) : "v"(p) : "memory");
    return r;
}
__device__ __forceinline__ void wait_ldv4(f4 &a, f4 &b, f4 &c)
{
    asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b), "+v"(c) : : "memory");
}
// x + (x of the lane that `ctrl` pairs this lane with), inside rows of 16 lanes
template <int CTRL> __device__ __forceinline__ float add_dpp(float x)
{
    return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, false));
}

// Workgroup barrier that first waits for every global access of this wavefront (loads,
// stores, no-return atomics) to be acknowledged.
__device__ __forceinline__ void wg_sync()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
}

// The same barrier where wavefront 0 (the dependent rounds) has nothing in flight that the
// others read: it does not wait for its stores of predictions to be acknowledged.
__device__ __forceinline__ void wg_sync_chain(int wave)
{
    if (wave != 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
}

#ifndef OCO_FOLD_LO
#define OCO_FOLD_LO 0x1p-100
#define OCO_FOLD_SOFT 0x1p-64
#endif
constexpr float kSparseFoldLoF = (float)(OCO_FOLD_LO);   // in-kernel emergency fold
constexpr double kSparseFoldSoft = OCO_FOLD_SOFT;  // fold between segments
#ifndef OCO_SEGMENT
#define OCO_SEGMENT 4096
#endif
constexpr int kSegment = OCO_SEGMENT;        // rounds per launch segment (absolute alignment)
constexpr int kWin = 64;                     // rounds per window (absolute alignment)
constexpr int kSpWaves = 16;                 // wavefronts per workgroup
constexpr int kBesideMaxWorkgroups = 128;    // window grids up to this size leave half the chip idle
constexpr size_t kLdsBytes = 160 * 1024;     // LDS of a gfx950 compute unit
constexpr int kMaxCross = 64;                // most round pairs across a window boundary that are corrected
constexpr int kProgBytes = 4096;             // head of the scratch: the window each workgroup has reached (one int each)
constexpr int kFetchMaxWorkgroups = 64;      // window grids up to this size get workgroups that fetch rows into L2 ahead of them
constexpr int kFetchAhead = 3;               // ... the rows of window x once every workgroup has reached window x - 3
constexpr int kFetchSpins = 4000;            // ... or after this many looks at the progress words (a hint never waits for good)

// (A build with -DOCO_SP_PROF keeps wall-clock sums (10 ns ticks) of the phases of workgroup 0's window loop in
// g_sp_prof -- eight entries per wavefront, wavefront 0 runs the dependent rounds -- read back
// through oco_debug_sp_prof: how the figures per phase in the comments below were taken.)
#ifdef OCO_SP_PROF
__device__ unsigned long long g_sp_prof[16 * 16 + 4];
#define SP_T(i) do { if (blockIdx.x == 0 && (threadIdx.x & 63) == 0) { const unsigned long long now_ = wall_clock64(); prof_[i] += now_ - last_; last_ = now_; } } while (0)
#else
#define SP_T(i) do { } while (0)
#endif

// Pre-pass over the round stream, one workgroup per window of the launch:
// G[s][t] = <x_s, x_t> for s < t, mask[s] = bit t set iff rounds s and t share a column,
// X2[t] = ||x_t||^2.  Window w of the launch covers rounds [wstart(w), wstart(w+1)).
struct WinPlan {
    int64_t t0;      // absolute round of the launch's first round
    int n;           // rounds in the launch
    __host__ __device__ int first_len() const { const int f = (int)(kWin - t0 % kWin); return f < n ? f : n; }
    __host__ __device__ int count() const { const int f = first_len(); return 1 + (n - f + kWin - 1) / kWin; }
    __host__ __device__ int start(int w) const { return w == 0 ? 0 : first_len() + (w - 1) * kWin; }
    __host__ __device__ int len(int w) const { const int s = start(w); const int l = w == 0 ? first_len() : kWin; return l < n - s ? l : n - s; }
};

// What the pre-pass leaves per window for the rounds kernel.
struct RoundRec {
    unsigned long long mask;            // bit t of round s: rounds s < t share a column
    double x2;                          // ||x_s||^2 (summed in float32)
};
struct WinRec {
    RoundRec rr[kWin];
    int off[kSpWaves + 1];              // phase C: wavefront c owns perm[off[c] .. off[c+1])
    int ng;                             // number of set mask bits
    unsigned any[2];                    // bit s: mask of round s is not empty
    int pad[32 - kSpWaves - 4];
    float g01[kWin];                    // <x_{t-1}, x_t> (optimistic update only; x_{-1}: previous call's last row)
    float x2h[kWin];                    // ||x_s||^2 / 2, as the dependent rounds read it
    int nx;                             // pairs (round s of the previous window, round t of this one) that share
    int padx[31];                       //   a column; -1: too many, or no previous window in this call
    unsigned short xs[kMaxCross], xt[kMaxCross];
    float xg[kMaxCross];                // their <x_s, x_t>, in (s, t) order
    unsigned short perm[kWin * OCO_MAX_NNZ];   // entries of the window sorted by column (stable); bit 15: column not unique
    float g[kWin * (kWin - 1) / 2];     // <x_s, x_t> of the set mask bits, in (s, t) order
};
static_assert(sizeof(WinRec) % 128 == 0, "window records stay 256-byte aligned");
constexpr int kRecHeadInts = (int)(offsetof(WinRec, perm) / 4);
// places in the head of a record (and of its copy in LDS), in ints
constexpr int kHeadOffs = (int)(offsetof(WinRec, off) / 4), kHeadAny = (int)(offsetof(WinRec, any) / 4);
constexpr int kHeadG01 = (int)(offsetof(WinRec, g01) / 4), kHeadX2 = (int)(offsetof(WinRec, x2h) / 4);
constexpr int kHeadCross = (int)(offsetof(WinRec, nx) / 4);
static_assert(kHeadOffs == 4 * kWin && kHeadG01 == 4 * kWin + 32 && kHeadCross == 4 * kWin + 32 + 2 * kWin, "record head layout");

__global__ void __launch_bounds__(1024) sparse_gram_kernel(const int32_t *col, const float *val, int nnz,
                                                          WinPlan plan, WinRec *recs, int optimistic,
                                                          const int32_t *last_col, const float *last_val, int shares, int wofs)
{
    __shared__ unsigned int xm[kWin][2];
    __shared__ int xrowoff[kWin + 1];
    __shared__ int cs[kWin * OCO_MAX_NNZ];
    __shared__ float vs[kWin * OCO_MAX_NNZ];
    __shared__ unsigned long long key[kWin * OCO_MAX_NNZ];      // (column, position), sorted in place
    __shared__ unsigned int mk[kWin][2];
    __shared__ int rowoff[kWin + 1];
    __shared__ unsigned short pair_s[kWin * (kWin - 1) / 2], pair_t[kWin * (kWin - 1) / 2];
    const int w = (int)blockIdx.x + wofs;
    const int ws = plan.start(w), wl = plan.len(w);
    const int total = wl * nnz;
    const unsigned mdiv = ((1u << 18) + nnz - 1) / nnz;       // e / nnz == (e * mdiv) >> 18 for e < 4096
    WinRec &rec = recs[w];
    for (int e = threadIdx.x; e < total; e += blockDim.x) {
        const int c = col[(int64_t)ws * nnz + e];
        cs[e] = c;
        vs[e] = val[(int64_t)ws * nnz + e];
        key[e] = ((unsigned long long)(unsigned)c << 12) | (unsigned)e;
    }
    // the previous window's entries are read where they lie (once each, but for the rare pairs)
    const int pws = w > 0 ? plan.start(w - 1) : 0, ptotal = w > 0 ? plan.len(w - 1) * nnz : 0;
    const int32_t *csp = col + (int64_t)pws * nnz;
    const float *vsp = val + (int64_t)pws * nnz;
    for (int e = threadIdx.x; e < kWin * 2; e += blockDim.x) { mk[e >> 1][e & 1] = 0u; xm[e >> 1][e & 1] = 0u; }
    __syncthreads();
    // sort by (column, position) -- a stable sort by column -- with a bitonic network over the
    // next power of two (padding keys are larger than any real key)
    int P = 2;
    while (P < total) P <<= 1;
    for (int e = total + threadIdx.x; e < P; e += blockDim.x) key[e] = ~0ull;
    __syncthreads();
    for (int k = 2; k <= P; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = threadIdx.x; i < P / 2; i += blockDim.x) {
                const int lo = ((i & ~(j - 1)) << 1) | (i & (j - 1));      // i with a zero inserted at bit log2(j)
                const int hi = lo | j;
                const unsigned long long a0 = key[lo], a1 = key[hi];
                const bool up = (lo & k) == 0;
                if ((a0 > a1) == up) { key[lo] = a1; key[hi] = a0; }
            }
            __syncthreads();
        }
    if (threadIdx.x < kWin) {
        float acc = 0.f;
        if (threadIdx.x < wl)
            for (int a = 0; a < nnz; ++a) acc = fmaf(vs[threadIdx.x * nnz + a], vs[threadIdx.x * nnz + a], acc);
        rec.rr[threadIdx.x].x2 = (double)acc;
        rec.x2h[threadIdx.x] = 0.5f * acc;
    }
    __syncthreads();
    // rounds that share a column sit next to each other in the sorted order
    for (int k = threadIdx.x; k < total; k += blockDim.x) {
        const unsigned long long kk = key[k];
        const int e = (int)(kk & 0xFFF);
        const unsigned long long c = kk >> 12;
        // bit 15: another entry of the window has the same column
        const bool dup = (k > 0 && (key[k - 1] >> 12) == c) || (k + 1 < total && (key[k + 1] >> 12) == c);
        rec.perm[k] = (unsigned short)(e | (dup ? 0x8000 : 0));
        const int s = (int)(((unsigned)e * mdiv) >> 18);
        for (int k2 = k + 1; k2 < total && (key[k2] >> 12) == c; ++k2) {
            const int t = (int)(((unsigned)(key[k2] & 0xFFF) * mdiv) >> 18);
            if (t > s) atomicOr(&mk[s][t >> 5], 1u << (t & 31));
        }
    }
    if (optimistic && threadIdx.x >= 64 && threadIdx.x < 64 + kWin) {
        // <x_{t-1}, x_t> for the hint of round t: the row before the window's first is the call's
        // previous row, or the row kept from the previous call
        const int t = threadIdx.x - 64;
        float g = 0.f;
        if (t < wl) {
            const int32_t *pc = t > 0 ? nullptr : (ws > 0 ? col + (int64_t)(ws - 1) * nnz : last_col);
            const float *pv = t > 0 ? nullptr : (ws > 0 ? val + (int64_t)(ws - 1) * nnz : last_val);
            for (int a2 = 0; a2 < nnz; ++a2) {
                const int ca = t > 0 ? cs[(t - 1) * nnz + a2] : pc[a2];
                const float va = t > 0 ? vs[(t - 1) * nnz + a2] : pv[a2];
                for (int b2 = 0; b2 < nnz; ++b2)
                    if (cs[t * nnz + b2] == ca) g = fmaf(va, vs[t * nnz + b2], g);
            }
        }
        rec.g01[t] = g;
    }
    if (threadIdx.x <= kSpWaves) {
        // equal shares of the sorted entries, cut only where the column changes
        const int sh = (int)threadIdx.x < shares ? (int)threadIdx.x : shares;
        int k = (int)((int64_t)sh * total / shares);
        while (k > 0 && k < total && (key[k] >> 12) == (key[k - 1] >> 12)) ++k;
        rec.off[threadIdx.x] = k;
    }
    // rounds of the previous window that share a column with a round of this one: look every
    // entry of the previous window up in the sorted list
    for (int ep = threadIdx.x; ep < ptotal; ep += blockDim.x) {
        const unsigned long long c = (unsigned long long)(unsigned)csp[ep];
        int lo = 0, hi = total;                                // first k with column(key[k]) >= c
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if ((key[mid] >> 12) < c) lo = mid + 1; else hi = mid;
        }
        const int s = (int)(((unsigned)ep * mdiv) >> 18);
        for (int k2 = lo; k2 < total && (key[k2] >> 12) == c; ++k2) {
            const int t = (int)(((unsigned)(key[k2] & 0xFFF) * mdiv) >> 18);
            atomicOr(&xm[s][t >> 5], 1u << (t & 31));
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int acc = 0;
        unsigned long long any = 0;
        for (int s2 = 0; s2 < kWin; ++s2) {
            rowoff[s2] = acc;
            acc += __popc(mk[s2][0]) + __popc(mk[s2][1]);
            if (mk[s2][0] | mk[s2][1]) any |= 1ull << s2;
        }
        rowoff[kWin] = acc;
        rec.ng = acc;
        rec.any[0] = (unsigned)any;
        rec.any[1] = (unsigned)(any >> 32);
        int xacc = 0;
        for (int s2 = 0; s2 < kWin; ++s2) {
            xrowoff[s2] = xacc;
            xacc += __popc(xm[s2][0]) + __popc(xm[s2][1]);
        }
        xrowoff[kWin] = xacc;
        rec.nx = (w == 0 || xacc > kMaxCross) ? -1 : xacc;
    }
    __syncthreads();
    if (w > 0 && xrowoff[kWin] <= kMaxCross && threadIdx.x >= 64 && threadIdx.x < 64 + kWin) {
        // one thread per round of the previous window: its pairs in order of t, each <x_s, x_t>
        // summed in a fixed order
        const int s2 = threadIdx.x - 64;
        unsigned long long m = (unsigned long long)xm[s2][0] | ((unsigned long long)xm[s2][1] << 32);
        int o = xrowoff[s2];
        while (m) {
            const int t = __builtin_ctzll(m);
            m &= m - 1;
            float g = 0.f;
            for (int a2 = 0; a2 < nnz; ++a2) {
                const int ca = csp[s2 * nnz + a2];
                for (int b2 = 0; b2 < nnz; ++b2)
                    if (cs[t * nnz + b2] == ca) g = fmaf(vsp[s2 * nnz + a2], vs[t * nnz + b2], g);
            }
            rec.xs[o] = (unsigned short)s2;
            rec.xt[o] = (unsigned short)t;
            rec.xg[o] = g;
            ++o;
        }
    }
    if (threadIdx.x < kWin) {
        const int s2 = threadIdx.x;
        unsigned long long m = (unsigned long long)mk[s2][0] | ((unsigned long long)mk[s2][1] << 32);
        rec.rr[s2].mask = m;
        int o = rowoff[s2];
        while (m) {
            const int t = __builtin_ctzll(m);
            m &= m - 1;
            pair_s[o] = (unsigned short)s2;
            pair_t[o] = (unsigned short)t;
            ++o;
        }
    }
    __syncthreads();
    // <x_s, x_t> of the pairs that share a column, each by one thread in a fixed order
    const int ng = rowoff[kWin];
    for (int o = threadIdx.x; o < ng; o += blockDim.x) {
        const int s2 = pair_s[o], t = pair_t[o];
        float g = 0.f;
        for (int a = 0; a < nnz; ++a) {
            const int ca = cs[s2 * nnz + a];
            for (int b = 0; b < nnz; ++b)
                if (cs[t * nnz + b] == ca) g = fmaf(vs[s2 * nnz + a], vs[t * nnz + b], g);
        }
        rec.g[o] = g;
    }
}

__device__ __forceinline__ int bcast_i(int v, int l) { return __builtin_amdgcn_readlane(v, l); }
__device__ __forceinline__ float bcast_f(float v, int l)
{
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}

// LDS of the rounds kernel that is staged per window, sized by the entries per round of the
// launch: cw | vw | head | perm2 | gl, each a multiple of 16 bytes.
constexpr int kGramInts = kWin * (kWin - 1) / 2;
__host__ __device__ inline int stage_perm_ints(int nnz) { return ((kWin * nnz + 1) / 2 + 3) & ~3; }
__host__ __device__ inline int stage_ints(int nnz) { return 2 * kWin * nnz + kRecHeadInts + stage_perm_ints(nnz) + kGramInts; }
struct WinStage {
    int *cw;
    float *vw;
    int *head;                                   // rr | off | ng | g01 | cross-window pairs (rr[kWin] may be read, never used)
    unsigned int *perm2;
    float *gl;
};
__device__ __forceinline__ WinStage stage_at(int *base, int nnz)
{
    WinStage st;
    st.cw = base;
    st.vw = reinterpret_cast<float *>(base + kWin * nnz);
    st.head = base + 2 * kWin * nnz;
    st.perm2 = reinterpret_cast<unsigned int *>(st.head + kRecHeadInts);
    st.gl = reinterpret_cast<float *>(st.head + kRecHeadInts + stage_perm_ints(nnz));
    return st;
}

// A window's stream entries and pre-pass record on their way into LDS, held in registers by
// the threads of at least 15 wavefronts: all loads are issued before the first is waited for
// (one memory round trip, not one per loop iteration; the trip counts are bounded by the sizes of
// the record), and other memory work can be issued between load() and store().
struct StageRegs {
    static constexpr int kMinThr = (kSpWaves - 1) * kWave;
    static constexpr int NE = (kWin * OCO_MAX_NNZ + kMinThr - 1) / kMinThr;
    static constexpr int NP = (kWin * OCO_MAX_NNZ / 2 + kMinThr - 1) / kMinThr;
    static constexpr int NG = (kGramInts + kMinThr - 1) / kMinThr;
    static constexpr int NH = (kRecHeadInts + kMinThr - 1) / kMinThr;
    int c[NE], h[NH];
    float x[NE], g[NG];
    unsigned int pp[NP];
    const int *ngp;

    __device__ __forceinline__ void load(const SparseArgs &a, const WinRec &rec, int ws, int total, int tid, int nthr)
    {
        const int nnz = a.nnz;
        const int *hsrc = reinterpret_cast<const int *>(&rec);
        const unsigned int *psrc = reinterpret_cast<const unsigned int *>(rec.perm);
        const int np = (total + 1) / 2;
        ngp = &rec.ng;
#pragma unroll
        for (int u = 0; u < NE; ++u) {
            const int e = tid + u * nthr;
            c[u] = e < total ? a.col[(int64_t)ws * nnz + e] : 0;
            x[u] = e < total ? a.val[(int64_t)ws * nnz + e] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < NH; ++u) {
            const int e = tid + u * nthr;
            h[u] = e < kRecHeadInts ? hsrc[e] : 0;
        }
#pragma unroll
        for (int u = 0; u < NP; ++u) {
            const int e = tid + u * nthr;
            pp[u] = e < np ? psrc[e] : 0u;
        }
#pragma unroll
        for (int u = 0; u < NG; ++u) {
            const int e = tid + u * nthr;
            g[u] = e < kGramInts ? rec.g[e] : 0.f;           // not gated by ng: no load waits for another
        }
    }
    __device__ __forceinline__ void store(const WinStage &st, int total, int tid, int nthr) const
    {
        const int np = (total + 1) / 2;
        const int ng = *ngp;
#pragma unroll
        for (int u = 0; u < NE; ++u) {
            const int e = tid + u * nthr;
            if (e < total) { st.cw[e] = c[u]; st.vw[e] = x[u]; }
        }
#pragma unroll
        for (int u = 0; u < NH; ++u) {
            const int e = tid + u * nthr;
            if (e < kRecHeadInts) st.head[e] = h[u];
        }
#pragma unroll
        for (int u = 0; u < NP; ++u) {
            const int e = tid + u * nthr;
            if (e < np) st.perm2[e] = pp[u];
        }
#pragma unroll
        for (int u = 0; u < NG; ++u) {
            const int e = tid + u * nthr;
            if (e < ng) st.gl[e] = g[u];
        }
    }
};

__device__ __forceinline__ void stage_window(const WinStage &st, const SparseArgs &a, const WinRec &rec, int ws, int total,
                                             int tid, int nthr)
{
    StageRegs sr;
    sr.load(a, rec, ws, total, tid, nthr);
    sr.store(st, total, tid, nthr);
}


// A workgroup owns LPW learners (LPW = 64, 32, 16, 8 or 4; fewer learners per workgroup spread a
// small problem over more compute units).  A wavefront is EPI = 64 / LPW slots of LPW lanes:
// lane = slot * LPW + learner, and one memory instruction touches EPI rows of V.
template <int LPW> struct Chain {
    float q0[kWin + 1][LPW];       // <v_start, x_t>, then corrected in place (row kWin: read ahead only)
    float yv[kWin + 1][LPW];       // labels
    float bw[kWin][LPW];           // step sizes b_t of the window
    float zb[kWin][LPW];           // predictions of the window, written to Z with the window's steps
};
// LDS the kernel declares itself, rounded up, and one chain buffer
constexpr int sparse_static_lds(int lpw) { return kSpWaves * lpw * 8 + lpw * 4 + 256; }
constexpr size_t sparse_chain_bytes(int lpw) { return (size_t)(2 * (kWin + 1) + 2 * kWin) * 4 * lpw; }
static_assert(sizeof(Chain<64>) == sparse_chain_bytes(64) && sizeof(Chain<4>) == sparse_chain_bytes(4), "chain buffer size");

// A staged window as the phases see it.
struct WinView {
    const int *cw;
    const float *vw;
    const RoundRec *rr;
    const int *offs;
    const int *any;
    const float *g01, *x2h;
    const int *xh;                 // nx | pad | xs | xt | xg
    const unsigned short *perm;
    const float *gl;
    int ws, wl;
};

// Where the LDS has room for it (pipe) the windows are pipelined: while wavefront 0 runs the
// dependent rounds of window w, the other fifteen first apply the steps of window w - 1 and
// stage window w + 1 and then, once those steps are in memory (the fifteen meet through a counter
// in LDS; wavefront 0 takes no part and goes on with its rounds), gather <v, x_t> for window w + 1.
// A workgroup barrier ends the window.  That gather sees V
// without the steps of window w; they enter as Gram terms over the window boundary,
//     <v_start(w+1), x_t> = <v_start(w), x_t> - sum_{s in w} b_s <x_s, x_t>,
// which the pre-pass lists (a handful of pairs for columns drawn at random).  The first window
// of a launch, a window with more than kMaxCross such pairs and the window after a fold inside
// the kernel are gathered after all earlier steps have been applied, as without the pipeline.
// Otherwise (64 learners per workgroup, or 64 entries per round with 32 learners) the LDS holds
// one set of buffers and every window runs gather, rounds, steps one after the other.
//
// A small problem leaves most compute units idle while each of its workgroups draws random rows of V
// through the one path from its compute unit to memory, which delivers a row that misses the L2 every
// ~1.5 ns against ~0.4 ns for a row that is there (measured; a window has 2048 of them to gather and as
// many to update).  The stream of columns is known in advance, so `nfetch` extra workgroups, one per
// XCD and L2, run ahead of the others and touch the rows of the coming windows: they load the bytes of
// every row that belong to the learners of their XCD and drop them.  They follow the progress words the
// working workgroups publish, with a bounded number of looks: being a hint, they never wait for good,
// and nothing waits for them.
template <int LOSS, int LPW, bool OPT>
__global__ void __launch_bounds__(kSpWaves *kWave) sparse_window_kernel(const SparseArgs a, WinPlan plan, int wbeg, int wend,
                                                                         int pipe, int nfetch)
{
    constexpr int EPI = kWave / LPW;
    constexpr int kCWaves = kSpWaves - 1;           // wavefronts that apply steps (all but the chain's)
    const bool PIPE = pipe != 0;
    const int NB = PIPE ? 2 : 1;                    // chain buffers: window w (, w + 1)
    extern __shared__ __align__(16) int smem_i[];   // NB chain buffers, then the staged windows (w - 1,) w, w + 1
    Chain<LPW> *chs = reinterpret_cast<Chain<LPW> *>(smem_i);
    int *stage0 = smem_i + NB * (int)(sizeof(Chain<LPW>) / 4);
    const int stage_n = stage_ints(a.nnz);
    auto stage_of = [&](int w) { return stage_at(stage0 + (PIPE ? (w - wbeg) % 3 : (w - wbeg) & 1) * stage_n, a.nnz); };
    // in-kernel fold: round after which the chain stopped (-1: none), the learners' scales, and
    // one partial squared norm per wavefront and learner
    __shared__ int fold_t, fold_gp, met;
    __shared__ float fold_sf[LPW];
    __shared__ double fold_part[kSpWaves][LPW];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l = lane % LPW, e = lane / LPW;       // learner and slot of this lane
#ifdef OCO_SP_PROF
    unsigned long long prof_[16] = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}, last_ = wall_clock64();
#endif
    const int nnz = a.nnz;
    const unsigned mdiv = ((1u << 18) + nnz - 1) / nnz;       // e / nnz == (e * mdiv) >> 18 for e < 4096
    // Workgroups go to the eight XCDs in turn, each with an L2 of its own: the workgroups of one
    // XCD take neighbouring learners, whose segments of a row of V share cache lines.
    const int nblk = (int)gridDim.x - nfetch;
    int *prog = static_cast<int *>(a.scratch);
    if ((int)blockIdx.x >= nblk) {
        // ---- a fetching workgroup (nfetch == 8, nblk % 8 == 0): XCD x = blockIdx - nblk holds the working
        // workgroups x, x + 8, ..., which own nblk / 8 * LPW neighbouring learners
        const int x = (int)blockIdx.x - nblk, ncx = nblk / 8;
        const int64_t base = (int64_t)x * ncx * LPW;          // first learner of the XCD
        const int lines = (ncx * LPW * 4 + 63) / 64;          // 64-byte pieces of a row to touch
#ifdef OCO_SP_PROF
        unsigned long long pf_[4] = {0, 0, 0, 0}, pl_ = wall_clock64();
#endif
        __shared__ int fetch_over;
        for (int w = wbeg + 1; w < wend; ++w) {
            if (threadIdx.x == 0) fetch_over = 0;
            if (threadIdx.x == 0 && w > wbeg + 2) {
                int m = 0;
                for (int spin = 0; spin < kFetchSpins; ++spin) {
                    m = 0x7fffffff;
                    for (int c = 0; c < ncx; ++c) {
                        const int v = __hip_atomic_load(prog + x + 8 * c, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        m = v < m ? v : m;
                    }
                    if (m >= w - kFetchAhead) break;
                    __builtin_amdgcn_s_sleep(32);
                }
                fetch_over = m >= wend - 1;                  // every working workgroup is in its last window: nothing left to fetch for
#ifdef OCO_SP_PROF
                pf_[2] += (unsigned long long)(w - m + 1000);
                pf_[3] += 1;
#endif
            }
#ifdef OCO_SP_PROF
            if (threadIdx.x == 0) { const unsigned long long n_ = wall_clock64(); pf_[0] += n_ - pl_; pl_ = n_; }
#endif
            __syncthreads();
            const bool over = fetch_over != 0;
            __syncthreads();                                 // (thread 0 writes the flag again in the next turn)
            if (over) break;
            const int ws = plan.start(w), total = plan.len(w) * a.nnz * lines;
            for (int e0 = threadIdx.x; e0 < total; e0 += 4 * (int)blockDim.x) {
                const float *pv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int e = e0 + u * (int)blockDim.x < total ? e0 + u * (int)blockDim.x : e0;
                    const int c = a.col[(int64_t)ws * a.nnz + e / lines];
                    pv[u] = a.V + (int64_t)c * a.RKp + base + (e % lines) * 16;
                }
                // The loaded words are dropped, but the registers they arrive in stay reserved until they have
                // arrived (the wait below names them): the compiler knows nothing of a load inside an asm
                // statement, and a register it gave to something else would be overwritten when the load returns.
                float got[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) asm volatile("global_load_dword %0, %1, off" : "=v"(got[u]) : "v"(pv[u]) : "memory");
                asm volatile("s_waitcnt vmcnt(0)" : "+v"(got[0]), "+v"(got[1]), "+v"(got[2]), "+v"(got[3]) : : "memory");
            }
#ifdef OCO_SP_PROF
            if (threadIdx.x == 0) { const unsigned long long n_ = wall_clock64(); pf_[1] += n_ - pl_; pl_ = n_; }
#endif
        }
#ifdef OCO_SP_PROF
        if (x == 0 && threadIdx.x == 0)
            for (int i2 = 0; i2 < 4; ++i2) atomicAdd(&g_sp_prof[16 * 16 + i2], pf_[i2]);
#endif
        return;
    }
    const int blk = nblk % 8 == 0 ? ((int)blockIdx.x % 8) * (nblk / 8) + (int)blockIdx.x / 8 : (int)blockIdx.x;
    const int q = blk * LPW + l;                    // learner (column of V) of this lane
    const unsigned uq = (unsigned)q;
    const int nq = a.R * a.K;
    const bool valid = q < nq;
    const int qq = valid ? q : 0;
    const int r = qq / a.K, i = qq % a.K;
    const float eta = valid ? a.eta[i] : 0.f;
    float *Vq = a.V + q;
    const float *yrow = a.y ? a.y + (int64_t)r * a.y_run_stride : nullptr;
    const unsigned zoff4 = 4u * (unsigned)(r * a.zl.zs_r + i * a.zl.zs_i);    // byte offset inside a round's slice of Z
    const int64_t zstep = 4 * a.zl.zs_t;
    const WinRec *recs = reinterpret_cast<const WinRec *>(static_cast<const char *>(a.scratch) + kProgBytes);
    // the lanes that run the dependent rounds (padding learners of the last workgroup take no part:
    // their step sizes stay zero and their scale stays one)
    const bool chain = wave == 0 && lane < LPW && valid;
    if (wave == 0 && lane < LPW && !valid) {
        for (int nb = 0; nb < NB; ++nb)
            for (int rd = 0; rd < kWin; ++rd) chs[nb].bw[rd][l] = 0.f;
    }
    if (wave == 0 && lane < LPW) fold_sf[l] = 1.f;
    double sigma0 = 1.0, n2 = 0.0;                  // n2: ||v||^2 as the state keeps it
    if (chain) { sigma0 = a.sigma[q]; n2 = a.n2[q]; }
    // Wait for these loads here.  Left to the compiler, the wait lands at their first use inside
    // the round loop, where it also waits for the previous round's store, every round.
    float eta_r = eta;
    asm volatile("" : "+v"(eta_r), "+v"(sigma0), "+v"(n2));
    const float eta2_r = 2.f * eta_r;
    double sigma = sigma0, hd = 0.5 * n2;           // the scale of w = sigma v, ||v||^2 / 2
    float sf = (float)sigma, isf = __builtin_amdgcn_rcpf(sf);
    const double Dhd = a.D * 0.70710678118654752440;   // D / sqrt(2)
    // optimistic update (Eq. (3)): hint ha * x_{t-1}, hp = <w^_t, x_{t-1}>, x2p = ||x_{t-1}||^2
    float ha = 0.f, hp = 0.f, x2p = 0.f;
    if (OPT && chain) { ha = a.ha[q]; hp = a.hp[q]; x2p = a.hx[q]; }
    if (OPT) asm volatile("" : "+v"(ha), "+v"(hp), "+v"(x2p));
    const float Df = (float)a.D, D2f = Df * Df;

    auto view = [&](int w) {
        const WinStage st = stage_of(w);
        WinView v;
        v.cw = st.cw;
        v.vw = st.vw;
        v.rr = reinterpret_cast<const RoundRec *>(st.head);
        v.offs = st.head + kHeadOffs;
        v.any = st.head + kHeadAny;
        v.g01 = reinterpret_cast<const float *>(st.head + kHeadG01);
        v.x2h = reinterpret_cast<const float *>(st.head + kHeadX2);
        v.xh = st.head + kHeadCross;
        v.perm = reinterpret_cast<const unsigned short *>(st.perm2);
        v.gl = st.gl;
        v.ws = plan.start(w);
        v.wl = plan.len(w);
        return v;
    };
    // ---- A: q0_t = <v, x_t> for the rounds of a window.  Wavefront wv of nwv takes the rounds
    // wv, wv + nwv, ..., RA at a time; slot e of the wavefront takes the entries j = e, e + EPI, ...
    // of a round -----------------------------------------------------------------------------
    auto gather_q0 = [&](auto ra_tag, auto bk_tag, const WinView &v, int wv, int nwv, float (*q0d)[LPW],
                         float (*yvd)[LPW]) {
        constexpr int RA = decltype(ra_tag)::value, BK = decltype(bk_tag)::value;   // RA * BK gathers in flight
        const int NL = (nnz + EPI - 1) / EPI;
        const int wl = v.wl;
        for (int tg = wv; tg < wl; tg += RA * nwv) {
            float acc[RA][4], yl[RA];
#pragma unroll
            for (int ra = 0; ra < RA; ++ra) {
                acc[ra][0] = acc[ra][1] = acc[ra][2] = acc[ra][3] = 0.f;
                const int t = tg + ra * nwv < wl ? tg + ra * nwv : tg;
                yl[ra] = yrow ? yrow[v.ws + t] : 0.f;               // in flight with the gathers
            }
            for (int k0 = 0; k0 < NL; k0 += BK) {
                float vv[RA][BK];
                int ci[RA][BK];
                // all columns of the batch first: one trip to LDS, not one per gather (the loads of V are
                // atomic loads, across which the compiler moves no other memory access)
#pragma unroll
                for (int ra = 0; ra < RA; ++ra) {
                    const int t = tg + ra * nwv < wl ? tg + ra * nwv : tg;
#pragma unroll
                    for (int u = 0; u < BK; ++u) {
                        const int j = (k0 + u) * EPI + e;
                        const bool in = k0 + u < NL && j < nnz;
                        ci[ra][u] = v.cw[t * nnz + (in ? j : 0)];
                    }
                }
#pragma unroll
                for (int ra = 0; ra < RA; ++ra)
#pragma unroll
                    for (int u = 0; u < BK; ++u) vv[ra][u] = ldv(a.V + (int64_t)ci[ra][u] * a.RKp + uq);
                SP_T(8);
#pragma unroll
                for (int ra = 0; ra < RA; ++ra) {
                    const int t = tg + ra * nwv < wl ? tg + ra * nwv : tg;
#pragma unroll
                    for (int u = 0; u < BK; ++u) {
                        const int j = (k0 + u) * EPI + e;
                        const bool in = k0 + u < NL && j < nnz;
                        const float xv = in ? v.vw[t * nnz + (in ? j : 0)] : 0.f;
                        acc[ra][u & 3] = fmaf(vv[ra][u], xv, acc[ra][u & 3]);
                    }
                }
                SP_T(9);
            }
#pragma unroll
            for (int ra = 0; ra < RA; ++ra) {
                const int t = tg + ra * nwv;
                float sum = (acc[ra][0] + acc[ra][1]) + (acc[ra][2] + acc[ra][3]);
#pragma unroll
                for (int sh = 32; sh >= LPW; sh >>= 1) sum += __shfl_xor(sum, sh);
                if (t < wl && lane < LPW) {
                    q0d[t][l] = sum;
                    yvd[t][l] = yl[ra];
                }
            }
        }
    };
    // The same for four learners per workgroup, where a row's share of the workgroup is 16 bytes: one lane
    // fetches them all, a round is the lanes of one instruction (nslot of them, two rounds per instruction
    // for 32 entries per round), and the sum over a round's entries is a butterfly over those lanes, the same
    // for every caller.  A quarter of the memory instructions of the form above.
    auto gather_q0_rows = [&](const WinView &v, int wv, int nwv, float (*q0d)[LPW], float (*yvd)[LPW], int pslot = 8) {
        (void)pslot;
        constexpr int NB = 3;                                // instructions in flight
        const int nslot = nnz <= 8 ? 8 : (nnz <= 16 ? 16 : (nnz <= 32 ? 32 : 64));
        const int rpi = kWave / nslot;                        // rounds per instruction
        const int j = lane & (nslot - 1), rsub = lane / nslot;
        const int wl = v.wl;
        const int ngroups = (wl + rpi - 1) / rpi;
        const float *Vb = a.V + (int64_t)blk * LPW;
        for (int g0 = wv; g0 < ngroups; g0 += NB * nwv) {
            int ci[NB];
            float xv[NB], yl[NB];
            f4 vv[NB];
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const int t = (g0 + u * nwv) * rpi + rsub;
                const bool in = t < wl && j < nnz;
                ci[u] = v.cw[in ? t * nnz + j : 0];
                xv[u] = v.vw[in ? t * nnz + j : 0];
            }
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const int t = (g0 + u * nwv) * rpi + rsub;
                vv[u] = ldv4(Vb + (int64_t)ci[u] * a.RKp);
                yl[u] = yrow && t < wl ? yrow[v.ws + t] : 0.f;
            }
            wait_ldv4(vv[0], vv[1], vv[2]);
            SP_T(pslot);
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const int t = (g0 + u * nwv) * rpi + rsub;
                const bool in = t < wl && j < nnz;
                const float xx = in ? xv[u] : 0.f;
                float pr[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    float x = __fmul_rn(vv[u][c], xx);       // (a product of its own: both lanes of a pair add the same two numbers)
                    x = add_dpp<0xB1>(x);                    // lanes ^ 1
                    x = add_dpp<0x4E>(x);                    // lanes ^ 2
                    x = add_dpp<0x141>(x);                   // the other quad of eight
                    pr[c] = x;
                }
                if (nslot >= 16) {
#pragma unroll
                    for (int c = 0; c < 4; ++c) pr[c] = add_dpp<0x140>(pr[c]);   // the other eight of sixteen
                }
                if (nslot >= 32) {
                    float o[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) o[c] = __shfl_xor(pr[c], 16);
#pragma unroll
                    for (int c = 0; c < 4; ++c) pr[c] += o[c];
                }
                if (nslot >= 64) {
                    float o[4];
#pragma unroll
                    for (int c = 0; c < 4; ++c) o[c] = __shfl_xor(pr[c], 32);
#pragma unroll
                    for (int c = 0; c < 4; ++c) pr[c] += o[c];
                }
                if (t < wl && j < 4) {
                    q0d[t][j] = j == 0 ? pr[0] : (j == 1 ? pr[1] : (j == 2 ? pr[2] : pr[3]));
                    yvd[t][j] = yl[u];
                }
            }
            SP_T(pslot + 1);
        }
    };
    // the predictions of a window go from LDS to Z (wavefronts 1 .. 15, a lane stores for its own learner)
    auto flush_z = [&](const WinView &v, const float (*zbp)[LPW]) {
        if (wave == 0 || !valid) return;
        char *zs = reinterpret_cast<char *>(a.Z) + zoff4;
        for (int t = (wave - 1) * EPI + e; t < v.wl; t += kCWaves * EPI)
            *reinterpret_cast<float *>(zs + (int64_t)(v.ws + t) * zstep) = zbp[t][l];
    };
    // ---- C: V[col] += -b_t x_t[col] for the rounds t <= tmax of a window, as no-return float
    // atomics.  All entries of a column belong to one wavefront (1 .. 15; wavefront 0 runs the
    // dependent rounds), which walks its share of the column-sorted list EPI entries per
    // instruction, so the adds to one address are issued in round order.  Entries of one column
    // that meet in an instruction are summed across slots first (fixed order); the pre-pass
    // marks them, and an instruction without any (nearly all, for columns drawn at random)
    // skips the exchange ------------------------------------------------------------------------
    auto apply_steps = [&](const WinView &v, const float (*bwp)[LPW], int tmax, auto partial) {   // partial: only t <= tmax
        if (wave == 0) return;
        const int beg = __builtin_amdgcn_readfirstlane(v.offs[wave - 1]);
        const int end = __builtin_amdgcn_readfirstlane(v.offs[wave]);
        constexpr int NI = 5;                                // instructions per batch
        for (int k0 = beg; k0 < end; k0 += NI * EPI) {
            int cc[NI];
            float xv[NI];
            bool dup[NI];
            // two trips to LDS per batch: the batch's places in the sorted list, then column, value and
            // step size of each (every read is in bounds: lanes past the share read its last entry, and the
            // empty asm keeps the compiler from putting a read under a branch of its own, one wait each)
            int pe[NI];
#pragma unroll
            for (int n = 0; n < NI; ++n) {
                const int k = k0 + n * EPI + e;
                pe[n] = v.perm[k < end ? k : end - 1];
            }
#pragma unroll
            for (int n = 0; n < NI; ++n) asm volatile("" : "+v"(pe[n]));
            float bl[NI];
#pragma unroll
            for (int n = 0; n < NI; ++n) {
                const int ee = pe[n] & 0xFFF;
                const int t = (int)(((unsigned)ee * mdiv) >> 18);
                cc[n] = v.cw[ee];
                xv[n] = v.vw[ee];
                bl[n] = bwp[t][l];
            }
#pragma unroll
            for (int n = 0; n < NI; ++n) asm volatile("" : "+v"(cc[n]), "+v"(xv[n]), "+v"(bl[n]));
#pragma unroll
            for (int n = 0; n < NI; ++n) {
                const bool act = k0 + n * EPI + e < end;
                const int t = (int)(((unsigned)(pe[n] & 0xFFF) * mdiv) >> 18);
                cc[n] = act ? cc[n] : -1;
                dup[n] = act && (pe[n] & 0x8000);
                xv[n] = act && (!decltype(partial)::value || t <= tmax) ? -bl[n] * xv[n] : 0.f;
            }
#pragma unroll
            for (int n = 0; n < NI; ++n) {
                bool last = true;
                if (EPI > 1 && __builtin_amdgcn_ballot_w64(dup[n]) != 0) {
#pragma unroll
                    for (int sh = 1; sh < EPI; sh <<= 1) {
                        const float ox = __shfl_up(xv[n], sh * LPW);
                        const int oc = __shfl_up(cc[n], sh * LPW);
                        if (e >= sh && oc == cc[n]) xv[n] += ox;
                    }
                    const int nc = __shfl_down(cc[n], LPW);
                    last = e == EPI - 1 || nc != cc[n];
                }
                if (cc[n] >= 0 && last) unsafeAtomicAdd(a.V + (int64_t)cc[n] * a.RKp + uq, xv[n]);
            }
        }
    };
    // The same for four learners per workgroup, where a row's share of the workgroup is 16 bytes: one lane
    // reads them, takes the step and writes them back.  A column that occurs once in the window is touched
    // by that lane alone between two barriers, so plain loads and stores do; the entries of a column that
    // occurs more than once stay with atomics, one lane at a time in the order of the sorted list (round
    // order).  Measured for the 2048 rows of a window: 2.4 us against 4.6 us with atomics, and rows that
    // were fetched ahead stay in L2, which they do not beside atomics.
    auto apply_rows = [&](const WinView &v, const float (*bwp)[LPW], int tmax, auto partial) {
        if (wave == 0) return;
        const int beg = __builtin_amdgcn_readfirstlane(v.offs[wave - 1]);
        const int end = __builtin_amdgcn_readfirstlane(v.offs[wave]);
        constexpr int NI = 3;                                // instructions per batch
        float *Vb = a.V + (int64_t)blk * LPW;
        for (int k0 = beg; k0 < end; k0 += NI * kWave) {
            int pe[NI];
#pragma unroll
            for (int n = 0; n < NI; ++n) {
                const int k = k0 + n * kWave + lane;
                pe[n] = v.perm[k < end ? k : end - 1];
            }
#pragma unroll
            for (int n = 0; n < NI; ++n) asm volatile("" : "+v"(pe[n]));
            int cc[NI];
            float xv[NI];
            f4 bl[NI];
#pragma unroll
            for (int n = 0; n < NI; ++n) {
                const int ee = pe[n] & 0xFFF;
                const int t = (int)(((unsigned)ee * mdiv) >> 18);
                cc[n] = v.cw[ee];
                xv[n] = v.vw[ee];
                bl[n] = *reinterpret_cast<const f4 *>(&bwp[t][0]);
            }
#pragma unroll
            for (int n = 0; n < NI; ++n) asm volatile("" : "+v"(cc[n]), "+v"(xv[n]), "+v"(bl[n]));
            float *row[NI];
            f4 cur[NI];
#pragma unroll
            for (int n = 0; n < NI; ++n) {
                row[n] = Vb + (int64_t)cc[n] * a.RKp;
                cur[n] = ldv4(row[n]);
            }
            wait_ldv4(cur[0], cur[1], cur[2]);
#pragma unroll
            for (int n = 0; n < NI; ++n) {
                const int t = (int)(((unsigned)(pe[n] & 0xFFF) * mdiv) >> 18);
                const bool act = k0 + n * kWave + lane < end && (!decltype(partial)::value || t <= tmax);
                const bool dup = (pe[n] & 0x8000) != 0;
                if (act && !dup) {
                    f4 nv;
#pragma unroll
                    for (int c = 0; c < 4; ++c) nv[c] = fmaf(-bl[n][c], xv[n], cur[n][c]);
                    *reinterpret_cast<f4 *>(row[n]) = nv;
                }
                unsigned long long dm = __builtin_amdgcn_ballot_w64(act && dup);
                while (dm) {
                    const int dl = __builtin_ctzll(dm);
                    dm &= dm - 1;
                    if (lane == dl) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) unsafeAtomicAdd(row[n] + c, -bl[n][c] * xv[n]);
                    }
                }
            }
        }
    };
    auto apply = [&](const WinView &v, const float (*bwp)[LPW], int tmax, auto partial) {
        if constexpr (LPW == 4) apply_rows(v, bwp, tmax, partial); else apply_steps(v, bwp, tmax, partial);
    };
    // ---- B: the dependent rounds tstart .. tstop - 1 of a window, scalars and LDS only (LPW
    // lanes of wavefront 0).  If a learner's sigma falls below the fold threshold the chain stops
    // after that round (fold_t), the whole workgroup folds and the chain goes on from the next
    // round.  gp: next Gram value of the window; returns the one after the rounds taken -----------
    // A round costs the wavefront that runs it about 7 clocks per instruction of the loop, whatever the
    // instruction (measured: 47 instructions 350 clocks, 40 instructions 278), so the loop is written for few
    // instructions.  With h = ||v||^2 / 2 in float64,
    //     ||v - b x||^2 / 2 = h + b (b ||x||^2 / 2 - <v, x>),
    // and the projection is sigma = min(sigma, D / ||v||) (||w|| = sigma ||v|| > D exactly when D / ||v|| < sigma):
    // sigma is taken afresh from ||v|| whenever the projection acts, so its rounding does not add up over the
    // rounds (a factor multiplied onto sigma round after round would let ||w|| drift off the sphere like a random
    // walk: 1.4e-5 after 1e5 rounds, measured).  The pre-pass leaves ||x||^2 / 2 for this.  The float64 minimum is
    // an instruction of its own: the compiler puts one more in front of it to quieten NaNs that cannot occur here
    // (|h| under the root: a sum that rounding took below zero projects nothing).
    auto run_chain = [&](const WinView &v, float (*q0)[LPW], const float (*yv)[LPW], float (*bw)[LPW], float (*zb)[LPW],
                         int tstart, int tstop, int gp) {
        const RoundRec *rr = v.rr;
        const float *gl = v.gl, *g01 = v.g01, *x2h = v.x2h;
        // rounds that share a column with a later round of the window (few): tc is the next of them
        unsigned long long any = (unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane(v.any[0]) |
                                 ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane(v.any[1]) << 32);
        any &= ~0ull << tstart;
        int tc = any ? __builtin_ctzll(any) : kWin;
        // one round; (qv, yy, xh): <v_t, x_t>, y_t, ||x_t||^2 / 2; (qn, yn, xn) receive those of the next round,
        // early.  True: a scale has fallen below the fold threshold and the rounds stop here.
        auto round = [&](int t, float qv, float yy, float xh, float &qn, float &yn, float &xn) -> bool {
            qn = q0[t + 1][l]; yn = yv[t + 1][l]; xn = x2h[t + 1];
            const float zr = sf * qv;                        // <w_t, x_t>
            float z = zr;
            if (OPT) {
                // played iterate w_t = s (w^_t - ha x_{t-1}), s from ||w^_t - ha x_{t-1}||^2: scalars only
                const float mf = fmaf(ha * ha, x2p, fmaf(-2.f * ha, hp, 2.f * (float)((sigma * sigma) * hd)));
                const float sp = mf > D2f ? Df * __builtin_amdgcn_rsqf(mf) : 1.f;
                z = sp * fmaf(-ha, g01[t], zr);
            }
            // for the squared loss eta * 2 (z - y) = (2 eta) (z - y) exactly
            const float step = LOSS == 1 ? eta2_r * (z - yy) : eta_r * slope<LOSS>(z, yy);
            const float b = step * isf;
            zb[t][l] = z;         // not to Z from here: a global store would queue behind the other wavefronts' memory work
            bw[t][l] = b;
            if (__builtin_expect(t == tc, 0)) {
                // (readfirstlane returns int: go through unsigned, or the low word sign-extends)
                const unsigned long long mk = rr[t].mask;
                unsigned long long m =
                    (unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)mk) |
                    ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(mk >> 32)) << 32);
                const bool next_hit = (m >> (t + 1)) & 1;
                while (m) {
                    const int t2 = __builtin_ctzll(m);
                    m &= m - 1;
                    q0[t2][l] = fmaf(-b, gl[gp++], q0[t2][l]);
                }
                if (next_hit) qn = q0[t + 1][l];
                any &= any - 1;
                tc = any ? __builtin_ctzll(any) : kWin;
            }
            hd = fma((double)b, (double)fmaf(b, xh, -qv), hd);
            asm("v_min_f64 %0, %1, %2" : "=v"(sigma) : "v"(sigma), "v"(Dhd * __builtin_amdgcn_rsq(__builtin_fabs(hd))));
            sf = (float)sigma;
            isf = __builtin_amdgcn_rcpf(sf);
            if (OPT) {                                      // next round's hint and <w^_{t+1}, x_t>
                hp = sf * fmaf(-b, 2.f * xh, qv);
                ha = step;
                x2p = 2.f * xh;
            }
            if (__builtin_expect(__any(sf < kSparseFoldLoF), 0)) {
                if (lane == 0) { fold_t = t; fold_gp = gp; }
                fold_sf[l] = sf;
                return true;
            }
            return false;
        };
        // four rounds per turn of the loop: the values read ahead alternate between two sets of registers
        float qa = q0[tstart][l], ya = yv[tstart][l], xa = x2h[tstart], qb, yb, xb;
        int t = tstart;
        for (; t + 4 <= tstop; t += 4) {
            if (round(t, qa, ya, xa, qb, yb, xb)) return gp;
            if (round(t + 1, qb, yb, xb, qa, ya, xa)) return gp;
            if (round(t + 2, qa, ya, xa, qb, yb, xb)) return gp;
            if (round(t + 3, qb, yb, xb, qa, ya, xa)) return gp;
        }
        for (; t < tstop; ++t) {
            if (round(t, qa, ya, xa, qb, yb, xb)) return gp;
            qa = qb; ya = yb; xa = xb;
        }
        return gp;
    };
    // A meeting of the wavefronts 1 .. 15 (not a workgroup barrier: wavefront 0 goes on with its rounds): each waits
    // for its own memory work, counts itself in LDS and waits until all fifteen of this meeting have.  Every one
    // of them comes to every meeting, so the wait ends.
    int meetings = 0;
    auto helpers_meet = [&]() {
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        ++meetings;
        if (lane == 0) __hip_atomic_fetch_add(&met, 1, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        while (__hip_atomic_load(&met, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP) < meetings * kCWaves) __builtin_amdgcn_s_sleep(2);
    };
    // What the wavefronts 1 .. 15 do beside the dependent rounds: the loads of window wn (on their
    // way into LDS) are issued first, then the steps and predictions of window wc, and only then
    // are the loads waited for; the next barrier waits for the atomics.
    auto work_beside = [&](int wn, bool steps, const WinView &vc, const float (*bwc)[LPW], const float (*zbc)[LPW]) {
        const int tid = (int)threadIdx.x - kWave;
        StageRegs sr;
        if (wn < wend) sr.load(a, recs[wn], plan.start(wn), plan.len(wn) * nnz, tid, kCWaves * kWave);
        SP_T(6);
        if (steps) { apply(vc, bwc, 0, std::false_type()); SP_T(7); flush_z(vc, zbc); }
        SP_T(10);
        if (wn < wend) sr.store(stage_of(wn), plan.len(wn) * nnz, tid, kCWaves * kWave);
    };

    // the dependent rounds are the critical path: their wavefront issues ahead of the three that
    // share its SIMD
    if (wave == 0) __builtin_amdgcn_s_setprio(3);
    stage_window(stage_of(wbeg), a, recs[wbeg], plan.start(wbeg), plan.len(wbeg) * nnz, threadIdx.x, blockDim.x);
    if (threadIdx.x == 0) { fold_t = -1; met = 0; }
    wg_sync();
    bool have_q0 = false;          // PIPE: this window's <v, x_t> were gathered beside the previous window's rounds
    bool pending = false;          // PIPE: the previous window's steps are not in V yet
    for (int w = wbeg; w < wend; ++w) {
        if (nfetch && threadIdx.x == kWave) __hip_atomic_store(prog + blockIdx.x, w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const WinView v = view(w);
        const int cb = PIPE ? (w - wbeg) & 1 : 0;
        Chain<LPW> &ch = chs[cb];                            // this window's buffers
        Chain<LPW> &cho = chs[cb ^ (NB - 1)];                // PIPE: the previous window's, then the next one's
        float (*q0)[LPW] = ch.q0;
        float (*yv)[LPW] = ch.yv;
        float (*bw)[LPW] = ch.bw;
        float (*zb)[LPW] = ch.zb;
        const int wl = v.wl;
        if (!have_q0) {
            if (PIPE && pending) {
                apply(view(w - 1), cho.bw, 0, std::false_type());
                flush_z(view(w - 1), cho.zb);
                wg_sync();
                pending = false;
            }
            if (LPW == 4)
                gather_q0_rows(v, wave, kSpWaves, q0, yv);
            else
                gather_q0(std::integral_constant<int, LPW == 64 ? 2 : 4>(),
                          std::integral_constant<int, LPW == 64 ? 16 : (LPW >= 16 ? 8 : (LPW == 8 ? 4 : 2))>(), v, wave,
                          kSpWaves, q0, yv);
            wg_sync();
        }
        int gp = 0;
        SP_T(0);
        if (PIPE) {
            // ---- the rounds of window w | steps of window w - 1 and staging of window w + 1, then, once
            // those steps are in memory (a meeting of the fifteen wavefronts only: the rounds go on),
            // <v, x_t> of window w + 1 (V holds the steps up to window w - 1) ----------------------
            if (wave == 0) {
                if (chain) {
                    if (have_q0) {
                        // steps of window w - 1 that the early gather has not seen
                        const int nx = v.xh[0];
                        const unsigned short *xs = reinterpret_cast<const unsigned short *>(v.xh + 32);
                        const unsigned short *xt = xs + kMaxCross;
                        const float *xg = reinterpret_cast<const float *>(v.xh + 32 + kMaxCross);
                        const float (*bwprev)[LPW] = cho.bw;
                        for (int p = 0; p < nx; ++p) q0[xt[p]][l] = fmaf(-bwprev[xs[p]][l], xg[p], q0[xt[p]][l]);
                    }
                    gp = run_chain(v, q0, yv, bw, zb, 0, wl, 0);
                }
                SP_T(1);
            } else {
                work_beside(w + 1, pending, pending ? view(w - 1) : v, cho.bw, cho.zb);
                SP_T(1);
                helpers_meet();
                SP_T(3);
            }
            if (wave != 0 && w + 1 < wend && stage_of(w + 1).head[kHeadCross] >= 0) {
                if (LPW == 4) {
                    gather_q0_rows(view(w + 1), wave - 1, kCWaves, cho.q0, cho.yv);
                } else
                    gather_q0(std::integral_constant<int, 5>(), std::integral_constant<int, LPW >= 16 ? 4 : (LPW == 8 ? 4 : 2)>(),
                              view(w + 1), wave - 1, kCWaves, cho.q0, cho.yv);
            }
            SP_T(4);
            wg_sync_chain(wave);
            SP_T(5);
            pending = false;
            have_q0 = w + 1 < wend && stage_of(w + 1).head[kHeadCross] >= 0;
        } else {
            if (chain) {
                run_chain(v, q0, yv, bw, zb, 0, wl, 0);
            } else if (wave != 0 && w + 1 < wend) {
                work_beside(w + 1, false, v, bw, zb);
            }
            wg_sync_chain(wave);
        }
        for (int ft = fold_t; ft >= 0; ft = fold_t) {
        const int gp0 = fold_gp;
        have_q0 = false;           // what was gathered for the next window is void after a fold
        // ---- fold inside the window (sigma below 2^-100 before the segment ended): apply the
        // steps taken so far, scale the workgroup's columns of V by sigma with all wavefronts,
        // measure ||v||^2 exactly, and take the remaining rounds' <v, x_t> afresh ----------------
        apply(v, bw, ft, std::true_type());
        wg_sync();
        {
            for (int rd = (int)threadIdx.x / LPW; rd <= ft; rd += kSpWaves * EPI) bw[rd][l] = 0.f;   // applied
            const float fs = fold_sf[l];
            const int64_t nslots = kSpWaves * EPI;
                double m2 = 0.0;
            for (int64_t j0 = wave * EPI + e; j0 < a.d; j0 += 4 * nslots) {
                float vv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int64_t j = j0 + u * nslots;
                    vv[u] = j < a.d ? ldv(Vq + j * a.RKp) : 0.f;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int64_t j = j0 + u * nslots;
                    const float wv = vv[u] * fs;
                    if (j < a.d) Vq[j * a.RKp] = wv;
                    m2 += (double)wv * (double)wv;
                }
            }
#pragma unroll
            for (int sh = 32; sh >= LPW; sh >>= 1) m2 += __shfl_xor(m2, sh);
            if (lane < LPW) fold_part[wave][l] = m2;
        }
        wg_sync();
        if (chain) {
            double m2 = 0.0;
            for (int wv = 0; wv < kSpWaves; ++wv) m2 += fold_part[wv][l];
            hd = 0.5 * m2;
            sigma = 1.0; sf = 1.f; isf = 1.f;
        }
        if (threadIdx.x == 0) fold_t = -1;
        if (LPW == 4)
            gather_q0_rows(v, wave, kSpWaves, q0, yv);
        else
            gather_q0(std::integral_constant<int, 1>(), std::integral_constant<int, 2>(), v, wave, kSpWaves, q0, yv);   // rare: few registers
        wg_sync();
        if (chain) run_chain(v, q0, yv, bw, zb, ft + 1, wl, gp0);
        wg_sync();
        }
        if (PIPE) {
            pending = true;                                  // applied beside the next window's rounds
        } else {
            apply(v, bw, 0, std::false_type());
            flush_z(v, zb);
            wg_sync();
        }
    }
    if (PIPE && pending) {
        apply(view(wend - 1), chs[(wend - 1 - wbeg) & 1].bw, 0, std::false_type());
        flush_z(view(wend - 1), chs[(wend - 1 - wbeg) & 1].zb);
        wg_sync();
    }
    if (chain) { a.sigma[q] = sigma; a.n2[q] = hd > 0.0 ? 2.0 * hd : 0.0; }
    if (OPT && chain) { a.ha[q] = ha; a.hp[q] = hp; a.hx[q] = x2p; }
#ifdef OCO_SP_PROF
    if (blockIdx.x == 0 && (threadIdx.x & 63) == 0)
        for (int i2 = 0; i2 < 16; ++i2) atomicAdd(&g_sp_prof[(threadIdx.x >> 6) * 16 + i2], prof_[i2]);
#endif
}

// Keeps the last round row of a call for the next call's first hint and for the export:
// first the old row is cleared from the dense copy, then the new one is written.
__global__ void __launch_bounds__(64) sparse_clear_last_kernel(const int32_t *last_col, float *xlast_dense, int nnz)
{
    if ((int)threadIdx.x < nnz) xlast_dense[last_col[threadIdx.x]] = 0.f;
}
__global__ void __launch_bounds__(64) sparse_keep_last_kernel(const int32_t *col, const float *val, int n, int nnz,
                                                              int32_t *last_col, float *last_val, float *xlast_dense)
{
    const int j = threadIdx.x;
    if (j >= nnz) return;
    const int c = col[(int64_t)(n - 1) * nnz + j];
    const float v = val[(int64_t)(n - 1) * nnz + j];
    last_col[j] = c;
    last_val[j] = v;
    xlast_dense[c] = v;
}

// z_u[r][t] = <u_t, x_t>: independent of the learners, one thread per (round, run)
__global__ void __launch_bounds__(256) sparse_comparator_kernel(const SparseArgs a)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= (int64_t)a.n * a.R) return;
    const int t = (int)(idx / a.R), r = (int)(idx % a.R);
    const int64_t tabs = a.t0 + t;
    int lo = 0, hi = a.S - 1;                     // last segment with seg_start <= tabs
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (a.seg_start[mid] <= tabs) lo = mid; else hi = mid - 1;
    }
    const float *uu = a.u + ((int64_t)r * a.S + lo) * a.d;
    const int32_t *ct = a.col + (int64_t)t * a.nnz;
    const float *vt = a.val + (int64_t)t * a.nnz;
    float acc = 0.f;
    for (int j = 0; j < a.nnz; ++j) acc = fmaf(uu[ct[j]], vt[j], acc);
    a.Z[(int64_t)r * a.zl.zs_r + (int64_t)a.K * a.zl.zs_i + (int64_t)t * a.zl.zs_t] = acc;
}

// Fold between segments: lane = column, one wavefront covers the 64 columns of a group.
__global__ void __launch_bounds__(256) sparse_fold_kernel(float *V, const double *sigma, int d, int RKp)
{
    const int lane = threadIdx.x & 63;
    const int q = blockIdx.y * kWave + lane;
    const double sg = sigma[q];
    if (!__any(sg < kSparseFoldSoft)) return;
    const float s = (float)sg;
    const int64_t stride = (int64_t)gridDim.x * 4;
    // eight rows in flight per wavefront (one at a time, the pass runs at a fraction of the memory's speed)
    for (int64_t j0 = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); j0 < d; j0 += 8 * stride) {
        float vv[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int64_t j = j0 + u * stride;
            vv[u] = j < d ? V[j * RKp + q] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int64_t j = j0 + u * stride;
            if (j < d) V[j * RKp + q] = vv[u] * s;
        }
    }
}

__global__ void __launch_bounds__(64) sparse_fold_finish_kernel(double *sigma, double *n2)
{
    const int q = blockIdx.x * kWave + threadIdx.x;
    const double sg = sigma[q];
    if (!__any(sg < kSparseFoldSoft)) return;
    const double sf = (double)(float)sg;          // the factor the columns were multiplied by
    n2[q] *= sf * sf;
    sigma[q] = 1.0;
}

}  // namespace

namespace {

// The largest share that still gives every compute unit a workgroup, at least 4.
int sparse_learners_per_workgroup(int nq, const Tuning &tune)
{
    int lpw = 64;
    {
        const int v = (int)tune.get(OCO_OPT_SPARSE_LPW);
        if (v == 4 || v == 8 || v == 16 || v == 32 || v == 64) return v;
    }
    while (lpw > 4 && (nq + lpw - 1) / lpw < 256) lpw >>= 1;
    return lpw;
}

template <int LOSS, int LPW, bool OPT>
hipError_t launch_window_lpw(const SparseArgs &a, const WinPlan &plan, int wbeg, int wend, hipStream_t s)
{
    const int nq = a.R * a.K;
    const int nblk = (nq + LPW - 1) / LPW;
    // fetching workgroups: one per XCD, where the grid is small, laid out by XCD (a multiple of 8) and a row's
    // share of an XCD is a few 64-byte pieces
    int nfetch = nblk % 8 == 0 && nblk <= kFetchMaxWorkgroups && wend - wbeg > 2 ? 8 : 0;
    if (a.tune->get(OCO_OPT_SPARSE_FETCH) == 0) nfetch = 0;
    const dim3 grid((unsigned)(nblk + nfetch)), block(kSpWaves * kWave);
    const size_t stage_b = (size_t)stage_ints(a.nnz) * 4, chain_b = sizeof(Chain<LPW>);
    // the pipelined kernel keeps two chain buffers and three staged windows
    int pipe = 2 * chain_b + 3 * stage_b + sparse_static_lds(LPW) <= kLdsBytes;
    if (a.tune->get(OCO_OPT_SPARSE_PIPE) == 0) pipe = 0;
    const size_t smem = pipe ? 2 * chain_b + 3 * stage_b : chain_b + 2 * stage_b;
    if (smem + sparse_static_lds(LPW) > kLdsBytes) return hipErrorInvalidValue;
    const auto kern = sparse_window_kernel<LOSS, LPW, OPT>;
    if (smem > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    hipError_t e = clock_begin(a.clock, s, "sparse_window_kernel");
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, block, smem, s, a, plan, wbeg, wend, pipe, nfetch);
    e = hipGetLastError();
    return e != hipSuccess ? e : clock_end(a.clock, s);
}

template <int LOSS, bool OPT>
hipError_t launch_window_loss(const SparseArgs &a, int lpw, const WinPlan &plan, int wbeg, int wend, hipStream_t s)
{
    switch (lpw) {
        case 64: return launch_window_lpw<LOSS, 64, OPT>(a, plan, wbeg, wend, s);
        case 32: return launch_window_lpw<LOSS, 32, OPT>(a, plan, wbeg, wend, s);
        case 16: return launch_window_lpw<LOSS, 16, OPT>(a, plan, wbeg, wend, s);
        case 8: return launch_window_lpw<LOSS, 8, OPT>(a, plan, wbeg, wend, s);
        case 4: return launch_window_lpw<LOSS, 4, OPT>(a, plan, wbeg, wend, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_window(const SparseArgs &a, int loss, int lpw, const WinPlan &plan, int wbeg, int wend, hipStream_t s)
{
    switch (loss) {
        case 0: return a.optimistic ? launch_window_loss<0, true>(a, lpw, plan, wbeg, wend, s)
                                    : launch_window_loss<0, false>(a, lpw, plan, wbeg, wend, s);
        case 1: return a.optimistic ? launch_window_loss<1, true>(a, lpw, plan, wbeg, wend, s)
                                    : launch_window_loss<1, false>(a, lpw, plan, wbeg, wend, s);
        case 2: return a.optimistic ? launch_window_loss<2, true>(a, lpw, plan, wbeg, wend, s)
                                    : launch_window_loss<2, false>(a, lpw, plan, wbeg, wend, s);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

#ifdef OCO_SP_PROF
extern "C" int oco_debug_sp_prof(unsigned long long *out, int clear)
{
    hipError_t e = hipMemcpyFromSymbol(out, HIP_SYMBOL(g_sp_prof), sizeof(unsigned long long) * 260);
    if (e == hipSuccess && clear) {
        unsigned long long z[260] = {0};
        e = hipMemcpyToSymbol(HIP_SYMBOL(g_sp_prof), z, sizeof z);
    }
    return (int)e;
}
#endif

size_t sparse_scratch_bytes(int64_t n_max)
{
    return kProgBytes + (size_t)(n_max / kWin + 2) * sizeof(WinRec);
}

hipError_t launch_sparse_rounds(const SparseArgs &a0, int loss, hipStream_t s, const PieceHook *hook)
{
    SparseArgs a = a0;
    if (a.n <= 0) return hipSuccess;
    if (a.nnz > OCO_MAX_NNZ) return hipErrorInvalidValue;

    // scratch: one record per window of the call
    const WinPlan plan{a.t0, a.n};
    const int nwin = plan.count();

    // segments end at the multiples of kSegment of the horizon, which are window boundaries
    const int groups = (a.R * a.K + kWave - 1) / kWave;
    int lpw = sparse_learners_per_workgroup(a.R * a.K, *a.tune);
    // one chain buffer and two staged windows have to fit the LDS (64 learners with more than 40
    // entries per round do not)
    while (lpw > 4 && sparse_chain_bytes(lpw) + 2 * (size_t)stage_ints(a.nnz) * 4 + sparse_static_lds(lpw) > kLdsBytes) lpw >>= 1;
    // the caller's per-segment work runs beside the following segments only while the window
    // kernel's workgroups leave at least half of the compute units idle
    if ((a.R * a.K + lpw - 1) / lpw > kBesideMaxWorkgroups) hook = nullptr;
    // The pre-pass of the first segment's windows goes ahead of the round kernels; that of the others runs beside
    // the first segment's rounds where the caller has a stream for it (the second launch then waits for it).
    WinRec *recs = reinterpret_cast<WinRec *>(static_cast<char *>(a.scratch) + kProgBytes);
    int nwin1 = 1;
    while (nwin1 < nwin && a.t0 + plan.start(nwin1) < (a.t0 / kSegment + 1) * kSegment) ++nwin1;
    const bool split = hook && hook->beside && hook->mark && hook->wait_mark && nwin1 < nwin;
    const int nfirst = split ? nwin1 : nwin;
    hipLaunchKernelGGL(sparse_gram_kernel, dim3(nfirst), dim3(1024), 0, s, a.col, a.val, a.nnz, plan, recs, a.optimistic,
                       a.last_col, a.last_val, kSpWaves - 1, 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    // the comparator's predictions feed the meta kernel only: beside the round kernels where
    // those leave room, else ahead of them
    {
        hipStream_t cs = s;
        if (hook && hook->beside) {
            e = hook->beside(hook->ctx, &cs);
            if (e != hipSuccess) return e;
        }
        if (split) {
            hipLaunchKernelGGL(sparse_gram_kernel, dim3(nwin - nfirst), dim3(1024), 0, cs, a.col, a.val, a.nnz, plan, recs,
                               a.optimistic, a.last_col, a.last_val, kSpWaves - 1, nfirst);
            e = hipGetLastError();
            if (e == hipSuccess) e = hook->mark(hook->ctx);
            if (e != hipSuccess) return e;
        }
        const int64_t nthr = (int64_t)a.n * a.R;
        hipLaunchKernelGGL(sparse_comparator_kernel, dim3((unsigned)((nthr + 255) / 256)), dim3(256), 0, cs, a);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    for (int wbeg = 0; wbeg < nwin;) {
        const int64_t seg_end = ((a.t0 + plan.start(wbeg)) / kSegment + 1) * kSegment;   // absolute
        int wend = wbeg + 1;
        while (wend < nwin && a.t0 + plan.start(wend) < seg_end) ++wend;
        if (split && wbeg == nfirst) {
            e = hook->wait_mark(hook->ctx);
            if (e != hipSuccess) return e;
        }
        e = launch_window(a, loss, lpw, plan, wbeg, wend, s);
        if (e != hipSuccess) return e;
        const int64_t reached = a.t0 + plan.start(wend - 1) + plan.len(wend - 1);
        if (hook) {
            const int off = plan.start(wbeg);
            e = hook->fn(hook->ctx, off, (int)(reached - a.t0) - off);
            if (e != hipSuccess) return e;
        }
        if (reached % kSegment == 0) {                        // a segment of the horizon ended
            hipLaunchKernelGGL(sparse_fold_kernel, dim3(1024, groups), dim3(256), 0, s, a.V, a.sigma, a.d, a.RKp);
            hipLaunchKernelGGL(sparse_fold_finish_kernel, dim3(groups), dim3(kWave), 0, s, a.sigma, a.n2);
        }
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        wbeg = wend;
    }
    if (a.optimistic) {
        hipLaunchKernelGGL(sparse_clear_last_kernel, dim3(1), dim3(64), 0, s, a.last_col, a.xlast_dense, a.nnz);
        hipLaunchKernelGGL(sparse_keep_last_kernel, dim3(1), dim3(64), 0, s, a.col, a.val, a.n, a.nnz, a.last_col,
                           a.last_val, a.xlast_dense);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace oco
