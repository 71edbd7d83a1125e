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
// (256 bytes for 64 learners), every gather and scatter is coalesced and all
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
// Per window the kernel therefore runs three phases:
//   A  all wavefronts: q0_t = <v_start, x_t> for the 64 rounds (bulk gathers);
//   B  one wavefront: the 64 dependent rounds on scalars and LDS only
//      (prediction, slope, step size b_t, norm, projection); the Gram terms
//      <x_r, x_t> come from a pre-pass over the round stream and are almost
//      all zero (two sparse rows rarely share a column); meanwhile the other
//      wavefronts stage the next window's stream and pre-pass record into a
//      second LDS buffer and pull its rows of V into L2;
//   C  all wavefronts: V[col] += -b_t x_t[col] as no-return float atomics, the
//      entries split over wavefronts by column so that the adds to one address
//      are issued by one wavefront in round order (bitwise reproducible).
//
// The comparator's predictions <u_t, x_t> do not depend on the learners and
// are taken by a separate, fully parallel kernel (one thread per run-round).
//
// On the boundary of the ball sigma shrinks geometrically (every projection
// multiplies it by a factor < 1) and v grows, so sigma has to be folded back
// into v now and then: V[:, q] *= sigma_q, ||v||^2 *= sigma_q^2, sigma_q = 1.
// The rounds are launched in segments that end at every 2048th round of the
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

// V is updated by float atomics, which execute in L2: every read of V in the window kernel
// goes to L2 as well (a device-scope relaxed load never hits in the per-CU cache).
__device__ __forceinline__ float ldv(const float *p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Workgroup barrier that first waits for every global access of this wavefront (loads,
// stores, no-return atomics) to be acknowledged.
__device__ __forceinline__ void wg_sync()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
}

#ifndef OCO_FOLD_LO
#define OCO_FOLD_LO 0x1p-100
#define OCO_FOLD_SOFT 0x1p-64
#endif
constexpr double kSparseFoldLo = OCO_FOLD_LO;    // in-kernel emergency fold
constexpr double kSparseFoldSoft = OCO_FOLD_SOFT;  // fold between segments
constexpr int kSegment = 2048;               // rounds per launch segment (absolute alignment)
constexpr int kWin = 64;                     // rounds per window (absolute alignment)
constexpr int kSpWaves = 16;                 // wavefronts per workgroup
constexpr int kBesideMaxWorkgroups = 128;    // window grids up to this size leave half the chip idle

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
    int pad[32 - kSpWaves - 2];
    float g01[kWin];                    // <x_{t-1}, x_t> (optimistic update only; x_{-1}: previous call's last row)
    unsigned short perm[kWin * OCO_MAX_NNZ];   // entries of the window sorted by column (stable)
    float g[kWin * (kWin - 1) / 2];     // <x_s, x_t> of the set mask bits, in (s, t) order
};
static_assert(sizeof(WinRec) % 128 == 0, "window records stay 256-byte aligned");
constexpr int kRecHeadInts = (int)(offsetof(WinRec, perm) / 4);

__global__ void __launch_bounds__(256) sparse_gram_kernel(const int32_t *col, const float *val, int nnz,
                                                          WinPlan plan, WinRec *recs, int optimistic,
                                                          const int32_t *last_col, const float *last_val)
{
    __shared__ int cs[kWin * OCO_MAX_NNZ];
    __shared__ float vs[kWin * OCO_MAX_NNZ];
    __shared__ unsigned long long key[kWin * OCO_MAX_NNZ];      // (column, position), sorted in place
    __shared__ unsigned int mk[kWin][2];
    __shared__ int rowoff[kWin + 1];
    __shared__ unsigned short pair_s[kWin * (kWin - 1) / 2], pair_t[kWin * (kWin - 1) / 2];
    const int w = blockIdx.x;
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
    for (int e = threadIdx.x; e < kWin * 2; e += blockDim.x) mk[e >> 1][e & 1] = 0u;
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
    }
    __syncthreads();
    // rounds that share a column sit next to each other in the sorted order
    for (int k = threadIdx.x; k < total; k += blockDim.x) {
        const unsigned long long kk = key[k];
        const int e = (int)(kk & 0xFFF);
        rec.perm[k] = (unsigned short)e;
        const unsigned long long c = kk >> 12;
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
        int k = (int)((int64_t)threadIdx.x * total / kSpWaves);
        while (k > 0 && k < total && (key[k] >> 12) == (key[k - 1] >> 12)) ++k;
        rec.off[threadIdx.x] = k;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int acc = 0;
        for (int s2 = 0; s2 < kWin; ++s2) {
            rowoff[s2] = acc;
            acc += __popc(mk[s2][0]) + __popc(mk[s2][1]);
        }
        rowoff[kWin] = acc;
        rec.ng = acc;
    }
    __syncthreads();
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

// LDS of the rounds kernel that is staged per window (two copies: the next window is
// staged while the dependent rounds of the current one run)
struct WinStage {
    int cw[kWin * OCO_MAX_NNZ];
    float vw[kWin * OCO_MAX_NNZ];
    int head[kRecHeadInts];                      // rr | off | ng (rr[kWin] may be read, never used)
    unsigned int perm2[kWin * OCO_MAX_NNZ / 2];
    float gl[kWin * (kWin - 1) / 2];
};

__device__ __forceinline__ void stage_window(WinStage &st, const SparseArgs &a, const WinRec &rec, int ws, int total,
                                             int tid, int nthr)
{
    const int ng = rec.ng;
    const int nnz = a.nnz;
    for (int e = tid; e < total; e += nthr) {
        st.cw[e] = a.col[(int64_t)ws * nnz + e];
        st.vw[e] = a.val[(int64_t)ws * nnz + e];
    }
    const int *hsrc = reinterpret_cast<const int *>(&rec);
    for (int e = tid; e < kRecHeadInts; e += nthr) st.head[e] = hsrc[e];
    const unsigned int *psrc = reinterpret_cast<const unsigned int *>(rec.perm);
    for (int e = tid; e < (total + 1) / 2; e += nthr) st.perm2[e] = psrc[e];
    for (int e = tid; e < ng; e += nthr) st.gl[e] = rec.g[e];
}

// 1/sqrt(x) for a finite x > 0: the hardware estimate (relative error < 6e-8, measured over
// [2^-200, 2^200]).  sigma is recomputed from ||v||^2 at every projection, so the error does not
// accumulate, and the iterate itself is float32.
__device__ __forceinline__ double rsqrt_pos(double x) { return __builtin_amdgcn_rsq(x); }

// A workgroup owns LPW learners (LPW = 64, 32, 16, 8 or 4; fewer learners per workgroup spread a
// small problem over more compute units).  A wavefront is EPI = 64 / LPW slots of LPW lanes:
// lane = slot * LPW + learner, and one memory instruction touches EPI rows of V.
template <int LPW> struct Chain {
    float q0[kWin + 1][LPW];       // <v_start, x_t>, then corrected in place (row kWin: read ahead only)
    float yv[kWin + 1][LPW];       // labels
    float bw[kWin][LPW];           // step sizes b_t of the window
};

template <int LOSS, int LPW, bool OPT>
__global__ void __launch_bounds__(kSpWaves *kWave) sparse_window_kernel(const SparseArgs a, WinPlan plan, int wbeg, int wend)
{
    constexpr int EPI = kWave / LPW;
    __shared__ Chain<LPW> ch;
    __shared__ __align__(16) WinStage stage[2];
    // in-kernel fold: round after which the chain stopped (-1: none), the learners' scales, and
    // one partial squared norm per wavefront and learner
    __shared__ int fold_t, fold_gp;
    __shared__ float fold_sf[LPW];
    __shared__ double fold_part[kSpWaves][LPW];

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int l = lane % LPW, e = lane / LPW;       // learner and slot of this lane
    const int nnz = a.nnz;
    const unsigned mdiv = ((1u << 18) + nnz - 1) / nnz;       // e / nnz == (e * mdiv) >> 18 for e < 4096
    const int q = blockIdx.x * LPW + l;             // learner (column of V) of this lane
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
    const double D2 = a.D * a.D;
    const WinRec *recs = static_cast<const WinRec *>(a.scratch);
    // the lanes that run the dependent rounds (padding learners of the last workgroup take no part:
    // their step sizes stay zero and their scale stays one)
    const bool chain = wave == 0 && lane < LPW && valid;
    if (wave == 0 && lane < LPW && !valid) {
        for (int rd = 0; rd < kWin; ++rd) ch.bw[rd][l] = 0.f;
    }
    if (wave == 0 && lane < LPW) fold_sf[l] = 1.f;
    double sigma = 1.0, n2 = 0.0;
    if (chain) { sigma = a.sigma[q]; n2 = a.n2[q]; }
    // Wait for these loads here.  Left to the compiler, the wait lands at their first use inside
    // the round loop, where it also waits for the previous round's store, every round.
    float eta_r = eta;
    asm volatile("" : "+v"(eta_r), "+v"(sigma), "+v"(n2));
    const float eta2_r = 2.f * eta_r;
    double sd2 = sigma * sigma;
    float sf = (float)sigma, isf = __builtin_amdgcn_rcpf(sf);
    // optimistic update (Eq. (3)): hint ha * x_{t-1}, hp = <w^_t, x_{t-1}>, x2p = ||x_{t-1}||^2
    float ha = 0.f, hp = 0.f, x2p = 0.f;
    if (OPT && chain) { ha = a.ha[q]; hp = a.hp[q]; x2p = a.hx[q]; }
    if (OPT) asm volatile("" : "+v"(ha), "+v"(hp), "+v"(x2p));
    const float Df = (float)a.D, D2f = Df * Df;

    stage_window(stage[0], a, recs[wbeg], plan.start(wbeg), plan.len(wbeg) * nnz, threadIdx.x, blockDim.x);
    if (threadIdx.x == 0) fold_t = -1;
    wg_sync();
    for (int w = wbeg; w < wend; ++w) {
        WinStage &st = stage[(w - wbeg) & 1];
        const int *cw = st.cw;
        const float *vw = st.vw;
        const RoundRec *rr = reinterpret_cast<const RoundRec *>(st.head);
        const int *offs = st.head + 4 * kWin;
        const float *g01 = reinterpret_cast<const float *>(st.head + 4 * kWin + 32);
        const unsigned short *perm = reinterpret_cast<const unsigned short *>(st.perm2);
        const float *gl = st.gl;
        const int ws = plan.start(w), wl = plan.len(w);
        // ---- A: q0_t = <v_start, x_t>; a wavefront takes rounds wave, wave + 16, ..., RA at a
        // time; slot e of the wavefront takes the entries j = e, e + EPI, ... of a round ----------
        auto gather_q0 = [&](auto ra_tag, auto bk_tag) {
            constexpr int RA = decltype(ra_tag)::value, BK = decltype(bk_tag)::value;   // RA * BK gathers in flight
            const int NL = (nnz + EPI - 1) / EPI;
            for (int tg = wave; tg < wl; tg += RA * kSpWaves) {
                float acc[RA][4], yl[RA];
#pragma unroll
                for (int ra = 0; ra < RA; ++ra) {
                    acc[ra][0] = acc[ra][1] = acc[ra][2] = acc[ra][3] = 0.f;
                    const int t = tg + ra * kSpWaves < wl ? tg + ra * kSpWaves : tg;
                    yl[ra] = yrow ? yrow[ws + t] : 0.f;             // in flight with the gathers
                }
                for (int k0 = 0; k0 < NL; k0 += BK) {
                    float vv[RA][BK];
#pragma unroll
                    for (int ra = 0; ra < RA; ++ra) {
                        const int t = tg + ra * kSpWaves < wl ? tg + ra * kSpWaves : tg;
#pragma unroll
                        for (int u = 0; u < BK; ++u) {
                            const int j = (k0 + u) * EPI + e;
                            const bool in = k0 + u < NL && j < nnz;
                            vv[ra][u] = ldv(a.V + (int64_t)cw[t * nnz + (in ? j : 0)] * a.RKp + uq);
                        }
                    }
#pragma unroll
                    for (int ra = 0; ra < RA; ++ra) {
                        const int t = tg + ra * kSpWaves < wl ? tg + ra * kSpWaves : tg;
#pragma unroll
                        for (int u = 0; u < BK; ++u) {
                            const int j = (k0 + u) * EPI + e;
                            const bool in = k0 + u < NL && j < nnz;
                            const float xv = in ? vw[t * nnz + (in ? j : 0)] : 0.f;
                            acc[ra][u & 3] = fmaf(vv[ra][u], xv, acc[ra][u & 3]);
                        }
                    }
                }
#pragma unroll
                for (int ra = 0; ra < RA; ++ra) {
                    const int t = tg + ra * kSpWaves;
                    float sum = (acc[ra][0] + acc[ra][1]) + (acc[ra][2] + acc[ra][3]);
#pragma unroll
                    for (int sh = 32; sh >= LPW; sh >>= 1) sum += __shfl_xor(sum, sh);
                    if (t < wl && lane < LPW) {
                        ch.q0[t][l] = sum;
                        ch.yv[t][l] = yl[ra];
                    }
                }
            }
        };
        // ---- C: V[col] += -b_t x_t[col] for the rounds t <= tmax.  All entries of a column belong
        // to one wavefront, which walks its share of the column-sorted list EPI entries per
        // instruction; entries of one column that meet in an instruction are summed across slots
        // first (fixed order) -------------------------------------------------------------------
        auto apply_steps = [&](int tmax, auto partial) {         // partial: only rounds t <= tmax (else all)
            const int beg = __builtin_amdgcn_readfirstlane(offs[wave]);
            const int end = __builtin_amdgcn_readfirstlane(offs[wave + 1]);
            constexpr int NI = 4;                                // instructions per batch
            for (int k0 = beg; k0 < end; k0 += NI * EPI) {
                int cc[NI];
                float xv[NI];
#pragma unroll
                for (int n = 0; n < NI; ++n) {
                    const int k = k0 + n * EPI + e;
                    const bool act = k < end;
                    const int ee = perm[act ? k : end - 1];
                    const int t = (int)(((unsigned)ee * mdiv) >> 18);
                    cc[n] = act ? cw[ee] : -1;
                    xv[n] = act && (!decltype(partial)::value || t <= tmax) ? -ch.bw[t][l] * vw[ee] : 0.f;
                }
#pragma unroll
                for (int n = 0; n < NI; ++n) {
                    bool last = true;
                    if (EPI > 1) {
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
        gather_q0(std::integral_constant<int, LPW == 64 ? 2 : 4>(),
                  std::integral_constant<int, LPW == 64 ? 16 : (LPW >= 16 ? 8 : (LPW == 8 ? 4 : 2))>());
        wg_sync();
        // ---- B: the dependent rounds, scalars and LDS only (LPW lanes of wavefront 0).  If a
        // learner's sigma falls below the fold threshold the chain stops after that round, the
        // whole workgroup folds (below) and the chain goes on from the next round ---------------
        auto run_chain = [&](int tstart, int gp) {               // gp: next Gram value of the window
            float qn = ch.q0[tstart][l], yn = ch.yv[tstart][l];
            RoundRec rn = rr[tstart];
            char *zs = reinterpret_cast<char *>(a.Z + (int64_t)(ws + tstart) * a.zl.zs_t);
            int tend = wl;                                       // a fold request ends the loop early
            for (int t = tstart; t < tend; ++t) {
                const float qv = qn, yy = yn;                    // <v_t, x_t>, y_t
                const RoundRec rc = rn;                          // collisions with later rounds, ||x_t||^2
                qn = ch.q0[t + 1][l]; yn = ch.yv[t + 1][l]; rn = rr[t + 1];        // next round, early
                float z = sf * qv;
                if (OPT) {
                    // played iterate w_t = s (w^_t - ha x_{t-1}), s from ||w^_t - ha x_{t-1}||^2: scalars only
                    const float mf = fmaf(ha * ha, x2p, fmaf(-2.f * ha, hp, (float)(sd2 * n2)));
                    const float sp = mf > D2f ? Df * __builtin_amdgcn_rsqf(mf) : 1.f;
                    z = sp * fmaf(-ha, g01[t], z);
                }
                *reinterpret_cast<float *>(zs + zoff4) = z;
                zs += zstep;
                // for the squared loss eta * 2 (z - y) = (2 eta) (z - y) exactly
                const float step = LOSS == 1 ? eta2_r * (z - yy) : eta_r * slope<LOSS>(z, yy);
                const float b = step * isf;
                ch.bw[t][l] = b;
                // (readfirstlane returns int: go through unsigned, or the low word sign-extends)
                unsigned long long m =
                    (unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)rc.mask) |
                    ((unsigned long long)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(rc.mask >> 32)) << 32);
                if (m) {
                    const bool next_hit = (m >> (t + 1)) & 1;
                    while (m) {
                        const int t2 = __builtin_ctzll(m);
                        m &= m - 1;
                        ch.q0[t2][l] = fmaf(-b, gl[gp++], ch.q0[t2][l]);
                    }
                    if (next_hit) qn = ch.q0[t + 1][l];
                }
                // ||v - b x||^2 = ||v||^2 + b (b ||x||^2 - 2 <v, x>)
                const double bd = (double)b;
                n2 = fma(bd, fma(bd, rc.x2, (double)(-2.f * qv)), n2);
                n2 = n2 > 0.0 ? n2 : 0.0;
                // projection: sigma = D / ||v||.  One select, then the values that follow from sigma
                // (the chain is bound by the number of instructions a single wavefront can issue)
                const double snew = a.D * rsqrt_pos(n2);
                sigma = n2 * sd2 > D2 ? snew : sigma;
                sd2 = sigma * sigma;
                sf = (float)sigma;
                isf = __builtin_amdgcn_rcpf(sf);
                if (OPT) {                                      // next round's hint and <w^_{t+1}, x_t>
                    hp = sf * fmaf(-b, (float)rc.x2, qv);
                    ha = step;
                    x2p = (float)rc.x2;
                }
                if (__any(sigma < kSparseFoldLo)) {
                    if (lane == 0) { fold_t = t; fold_gp = gp; }
                    fold_sf[l] = sf;
                    tend = t + 1;
                }
            }
        };
        if (chain) {
            run_chain(0, 0);
        } else if (wave != 0 && w + 1 < wend) {
            // ---- meanwhile the other wavefronts stage the next window -------------------------
            stage_window(stage[(w + 1 - wbeg) & 1], a, recs[w + 1], plan.start(w + 1), plan.len(w + 1) * nnz,
                         (int)threadIdx.x - kWave, (kSpWaves - 1) * kWave);
            if (a.prefetch) {
                // ... and pull its rows of V towards L2 (one lane per row segment of this workgroup)
                const int ns = plan.start(w + 1), ntot = plan.len(w + 1) * nnz;
                float sink = 0.f;
                for (int en = (int)threadIdx.x - kWave; en < ntot; en += (kSpWaves - 1) * kWave)
                    sink += ldv(a.V + (int64_t)a.col[(int64_t)ns * nnz + en] * a.RKp + blockIdx.x * LPW);
                if (sink == 1.2345e30f) a.Z[0] = sink;          // never true; keeps the loads alive
            }
        }
        wg_sync();
        for (int ft = fold_t; ft >= 0; ft = fold_t) {
        const int gp0 = fold_gp;
        // ---- fold inside the window (sigma below 2^-100 before the segment ended): apply the
        // steps taken so far, scale the workgroup's columns of V by sigma with all wavefronts,
        // measure ||v||^2 exactly, and take the remaining rounds' <v, x_t> afresh ----------------
        apply_steps(ft, std::true_type());
        wg_sync();
        {
            for (int rd = (int)threadIdx.x / LPW; rd <= ft; rd += kSpWaves * EPI) ch.bw[rd][l] = 0.f;   // applied
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
            n2 = m2;
            sigma = 1.0; sd2 = 1.0; sf = 1.f; isf = 1.f;
        }
        if (threadIdx.x == 0) fold_t = -1;
        gather_q0(std::integral_constant<int, 1>(), std::integral_constant<int, 2>());   // rare: few registers
        wg_sync();
        if (chain) run_chain(ft + 1, gp0);
        wg_sync();
        }
        apply_steps(wl - 1, std::false_type());
        wg_sync();
    }
    if (chain) { a.sigma[q] = sigma; a.n2[q] = n2; }
    if (OPT && chain) { a.ha[q] = ha; a.hp[q] = hp; a.hx[q] = x2p; }
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
    for (int64_t j = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6); j < d; j += stride)
        V[j * RKp + q] *= s;
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
int sparse_learners_per_workgroup(int nq)
{
    int lpw = 64;
    if (const char *f = getenv("OCO_SPARSE_LPW")) {
        const int v = atoi(f);
        if (v == 4 || v == 8 || v == 16 || v == 32 || v == 64) return v;
    }
    while (lpw > 4 && (nq + lpw - 1) / lpw < 256) lpw >>= 1;
    return lpw;
}

template <int LOSS, bool OPT>
hipError_t launch_window_loss(const SparseArgs &a, int lpw, const WinPlan &plan, int wbeg, int wend, hipStream_t s)
{
    const int nq = a.R * a.K;
    const dim3 grid((unsigned)((nq + lpw - 1) / lpw)), block(kSpWaves * kWave);
    switch (lpw) {
        case 64: hipLaunchKernelGGL((sparse_window_kernel<LOSS, 64, OPT>), grid, block, 0, s, a, plan, wbeg, wend); break;
        case 32: hipLaunchKernelGGL((sparse_window_kernel<LOSS, 32, OPT>), grid, block, 0, s, a, plan, wbeg, wend); break;
        case 16: hipLaunchKernelGGL((sparse_window_kernel<LOSS, 16, OPT>), grid, block, 0, s, a, plan, wbeg, wend); break;
        case 8: hipLaunchKernelGGL((sparse_window_kernel<LOSS, 8, OPT>), grid, block, 0, s, a, plan, wbeg, wend); break;
        case 4: hipLaunchKernelGGL((sparse_window_kernel<LOSS, 4, OPT>), grid, block, 0, s, a, plan, wbeg, wend); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
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

size_t sparse_scratch_bytes(int64_t n_max)
{
    return (size_t)(n_max / kWin + 2) * sizeof(WinRec);
}

hipError_t launch_sparse_rounds(const SparseArgs &a0, int loss, hipStream_t s, const PieceHook *hook)
{
    SparseArgs a = a0;
    if (a.n <= 0) return hipSuccess;
    if (a.nnz > OCO_MAX_NNZ) return hipErrorInvalidValue;
    const int64_t nthr = (int64_t)a.n * a.R;
    hipLaunchKernelGGL(sparse_comparator_kernel, dim3((unsigned)((nthr + 255) / 256)), dim3(256), 0, s, a);

    // scratch: one record per window of the call
    const WinPlan plan{a.t0, a.n};
    const int nwin = plan.count();
    hipLaunchKernelGGL(sparse_gram_kernel, dim3(nwin), dim3(256), 0, s, a.col, a.val, a.nnz, plan,
                       static_cast<WinRec *>(a.scratch), a.optimistic, a.last_col, a.last_val);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;

    // segments end at the multiples of kSegment of the horizon, which are window boundaries
    const int groups = a.RKp / kWave;
    const int lpw = sparse_learners_per_workgroup(a.R * a.K);
    // the caller's per-segment work runs beside the following segments only while the window
    // kernel's workgroups leave at least half of the compute units idle
    if ((a.R * a.K + lpw - 1) / lpw > kBesideMaxWorkgroups) hook = nullptr;
    for (int wbeg = 0; wbeg < nwin;) {
        const int64_t seg_end = ((a.t0 + plan.start(wbeg)) / kSegment + 1) * kSegment;   // absolute
        int wend = wbeg + 1;
        while (wend < nwin && a.t0 + plan.start(wend) < seg_end) ++wend;
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
