// Dense rounds of the base learners (Sec. 3.1 update inside the ensemble of
// Sec. 3.3), many rounds per launch.
//
// Mapping.  One wavefront owns one base learner of one run for the whole call:
// lane l keeps d/64 coordinates of the iterate in registers, so the inner
// product <w_t^i, x_t> and the norm of the stepped vector are wavefront
// reductions (DPP) and no learner ever waits for another -- each base learner
// steps along the gradient at its own iterate.  One extra wavefront per run
// carries the comparator u_t and only takes inner products.  The wavefronts of
// a workgroup share the round stream: x is copied from global memory straight
// into an LDS ring of three tiles of RT rounds (global_load_lds, no staging
// registers), two tiles ahead of the compute, one barrier per tile.
//
// One pass over the registers per round.  The iterate is kept as w = sigma*v
// with a per-learner scalar sigma, so the projection onto the ball only
// changes sigma.  In round t the pass computes
//     v      <- v - b x_t,  b = eta c_t / sigma    (gradient step, c_t = phi'(z_t; y_t))
//     q      =  <v, x_{t+1}>                       (next round's prediction)
// and the norm needed by the projection follows from scalars already at hand,
//     ||v - b x_t||^2 = ||v||^2 - 2 b <v, x_t> + b^2 ||x_t||^2
// (<v, x_t> is the previous round's q, ||x_t||^2 comes from a small pre-pass
// over the round stream), carried in float32 like its inputs (float64 for the
// three scalars changed no result: the error is that of <v, x_t>) and
// re-measured exactly, as sum_j v_j^2 inside the pass, at every 64th round of
// the horizon so that rounding cannot accumulate.  Then sigma <- D/||v|| if sigma ||v|| > D, and
// z_{t+1} = sigma q.  x_{t+1} is
// read from LDS during the pass, one chunk ahead of the arithmetic, and stays
// in registers as the next round's x_t (two register sets that swap roles, the
// round loop is unrolled by two).  sigma is folded back into v, at the start of
// a round, once it has left [2^-24, 2^24].
//
// The kernel writes z_t^i for every round to Z; losses, Hedge weights and
// regret are computed from Z by the meta kernel.
#include "oco_internal.h"
#include "../../include/oco.h"

#include <algorithm>
#include <cstdio>
#include <cstdlib>

namespace oco {
namespace {

template <int NPL> struct DenseCfg;
// NPL: coordinates per lane.  MAXW: most wavefronts per workgroup (sets the register
// budget).  RT: rounds per LDS tile (even; RT*NPL a multiple of 4).
template <> struct DenseCfg<1>  { static constexpr int MAXW = 16, RT = 32; };
template <> struct DenseCfg<2>  { static constexpr int MAXW = 16, RT = 16; };
template <> struct DenseCfg<4>  { static constexpr int MAXW = 16, RT = 16; };
template <> struct DenseCfg<8>  { static constexpr int MAXW = 16, RT = 8; };
#ifndef OCO_RT16
#define OCO_RT16 2
#endif
template <> struct DenseCfg<16> { static constexpr int MAXW = 16, RT = OCO_RT16; };
#ifndef OCO_MAXW32
#define OCO_MAXW32 12
#endif
template <> struct DenseCfg<32> { static constexpr int MAXW = OCO_MAXW32, RT = 2; };
#ifndef OCO_MAXW64
#define OCO_MAXW64 12
#endif
template <> struct DenseCfg<64> { static constexpr int MAXW = OCO_MAXW64,  RT = 2; };
// One register set for the round row (x_t is replaced chunk by chunk with x_{t+1} as the step
// consumes it) instead of two that swap roles: 64 fewer registers per lane, which at 64
// coordinates per lane is the difference between two and three wavefronts per SIMD.
template <int NPL> constexpr bool kOneRowSet = NPL >= 64;   // at 32 it measured 4 % slower
constexpr int kRing = 3;   // LDS tiles
constexpr int64_t kStreamPieceBytes = 64ll << 20;  // shared round stream per launch of a multi-pass grid
constexpr int64_t kPieceMinRounds = 512;           // no piece shorter than this
constexpr int64_t kBesideMaxWaves = 1024;          // one wavefront per SIMD: the chip is mostly idle
constexpr int64_t kBesidePieces = 4;
constexpr int64_t kHalfMinTasks = 8192;           // two learners per wavefront from this many learners on:
                                                   // four wavefronts per SIMD (with 4352 it measured 13 % slower)

template <int VW> struct VecT;
template <> struct VecT<1> { using type = float; };
template <> struct VecT<2> { using type = float2; };
template <> struct VecT<4> { using type = float4; };

template <int VW> __device__ __forceinline__ void unpack(const typename VecT<VW>::type &t, float (&o)[VW])
{
    if constexpr (VW == 4) { o[0] = t.x; o[1] = t.y; o[2] = t.z; o[3] = t.w; }
    else if constexpr (VW == 2) { o[0] = t.x; o[1] = t.y; }
    else { o[0] = t; }
}

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_term(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}

// Sum over the 64 lanes, result uniform.  Fixed order: xor-butterfly inside each row of
// 16 lanes, then rows 0+1 and 2+3, then the two halves.  The two cross-row steps are
// written as v_add_f32 with a DPP row broadcast and a row mask: rows outside the mask keep
// their value, so one instruction does what mov+mov_dpp+add would.  (A DPP operand needs
// two wait states after the VALU write that produced it, hence the s_nop.)
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_term<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
    v += dpp_term<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
    v += dpp_term<0x141, 0xF>(v);   // row_half_mirror
    v += dpp_term<0x140, 0xF>(v);   // row_mirror
    asm("s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"   // rows 1, 3 += row 0, 2
        "s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"   // rows 2, 3 += rows 0+1
        "s_nop 0"
        : "+v"(v));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ __forceinline__ float fast_rcp(float x) { return __builtin_amdgcn_rcpf(x); }

// Workgroup barrier that publishes the tiles copied global -> LDS.  Those copies complete
// asynchronously and are counted by vmcnt of the wavefront that issued them; a plain barrier
// does not wait for them (a workgroup-scope fence leaves vmcnt alone), and a wavefront that never
// reads the ring (padding wavefronts) would otherwise meet the barrier with its share of a tile
// still in flight.  Every wavefront therefore drains its own copies before it arrives.
__device__ __forceinline__ void tile_sync()
{
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
}

template <int LOSS> __device__ __forceinline__ float slope(float z, float y)
{
    if (LOSS == 0) return 1.0f;
    if (LOSS == 1) return 2.0f * (z - y);
    // logistic: -y / (1 + exp(y z)); exp overflow gives -y * (1/inf) = -0
    return -y * fast_rcp(1.0f + __expf(y * z));
}

template <int VW> __device__ __forceinline__ float combine(const float (&acc)[VW])
{
    if (VW == 4) return (acc[0] + acc[1]) + (acc[2] + acc[3]);
    if (VW == 2) return acc[0] + acc[1];
    return acc[0];
}

template <int NPL, int LOSS, bool OPT>
__global__ void __launch_bounds__(DenseCfg<NPL>::MAXW * kWave)
dense_rounds_kernel(const DenseArgs a)
{
    using C = DenseCfg<NPL>;
    constexpr int VW = NPL >= 4 ? 4 : NPL;      // floats per LDS read
    constexpr int NV = NPL / VW;                // LDS reads per lane and round
    constexpr int DP = NPL * kWave;             // padded dimension
    constexpr int RT = C::RT;
    constexpr int TILE = RT * DP;               // floats per tile
    constexpr int RING_ROUNDS = kRing * RT;
    constexpr int NI = TILE / 4 / kWave;        // 1 KB copy instructions per tile
    constexpr int CH = NV >= 2 ? 2 : 1;         // LDS reads per chunk
#ifndef OCO_NACC64
#define OCO_NACC64 4
#endif
    // partial sums of the next-round dot: two chains (one add to combine them), four where the
    // chains would get 32 FMAs long
    constexpr int NACC = NPL >= 64 ? OCO_NACC64 : (VW >= 2 ? 2 : 1);
    constexpr int NCH = NV / CH;
    static_assert(TILE % (4 * kWave) == 0, "tile must be a whole number of 1 KB copies");
    static_assert(RT % 2 == 0, "the round loop is unrolled by two");
    using V = typename VecT<VW>::type;

    extern __shared__ float4 smem4[];
    float *ring = reinterpret_cast<float *>(smem4);

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    const int wpb = nthreads >> 6;              // wavefronts in this workgroup
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = a.n;
    const int d = a.d;
    const int K = a.K;

    // ---- which task this wavefront owns: learner i < K, or the comparator (i == K) ----
    int r, i;
    bool active;
    if (a.x_shared) {
        const int64_t q = (int64_t)blockIdx.x * wpb + wave;
        active = q < (int64_t)a.R * a.per_run;
        r = active ? (int)(q / a.per_run) : 0;
        i = active ? (int)(q % a.per_run) : 0;
    } else {
        r = blockIdx.y;
        i = blockIdx.x * wpb + wave;
        active = i < a.per_run;
        if (!active) i = 0;
    }
    const bool is_cmp = active && i == K;
    const float *xg = a.x_shared ? a.x : a.x + (int64_t)blockIdx.y * a.x_run_stride;

    // ---- staging of x: tile k = rounds k*RT .. k*RT+RT-1 -> ring slot k % 3 ------
    auto issue_tile = [&](int k) {
        float *dst = ring + (k % kRing) * TILE;
        if (a.vec_ok) {
            for (int ii = wave; ii < NI; ii += wpb) {
                const int e = ii * kWave + lane;               // float4 index in the tile
                const int rr = e / (DP / 4), j4 = e % (DP / 4);
                const int tt = k * RT + rr;
                if (tt < n && j4 * 4 < d)
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void *)(xg + (int64_t)tt * d + j4 * 4),
                        (__attribute__((address_space(3))) void *)(dst + ii * 4 * kWave), 16, 0, 0);
            }
        } else {                                               // any d, any alignment
            for (int e = tid; e < TILE; e += nthreads) {
                const int rr = e / DP, j = e % DP;
                const int tt = k * RT + rr;
                if (tt < n && j < d) dst[e] = xg[(int64_t)tt * d + j];
            }
        }
    };

    // padding coordinates (j >= d) of the ring are never written again: zero them once
    for (int e = tid; e < kRing * TILE / 4; e += nthreads) smem4[e] = make_float4(0.f, 0.f, 0.f, 0.f);
    tile_sync();
    const int ntiles = (n + RT - 1) / RT;
    issue_tile(0);
    if (ntiles > 1) issue_tile(1);
    tile_sync();

    auto xrow = [&](int t) { return reinterpret_cast<const V *>(ring + (t % RING_ROUNDS) * DP); };
    const float *yrow = a.y ? a.y + (int64_t)r * a.y_run_stride : nullptr;

    // Each role runs its own copy of the tile loop (same number of barriers in each), so
    // that the register-resident vector of one role never meets another role's code.
    if (!active) {
        for (int k = 0; k < ntiles; ++k) {
            if (k + 2 < ntiles) issue_tile(k + 2);
            tile_sync();
        }
        return;
    }

    if (is_cmp) {
        // ---- comparator wavefront: z_t = <u_t, x_t>, no step -----------------------------
        float uv[NV][VW];
        auto load_u = [&](int sg) {
            const float *src = a.u + ((int64_t)r * a.S + sg) * d;
#pragma unroll
            for (int m = 0; m < NV; ++m)
#pragma unroll
                for (int e = 0; e < VW; ++e) {
                    const int j = (m * kWave + lane) * VW + e;
                    uv[m][e] = j < d ? src[j] : 0.f;
                }
        };
        auto dot_u = [&](const V *xr) {
            float acc[VW];
#pragma unroll
            for (int e = 0; e < VW; ++e) acc[e] = 0.f;
#pragma unroll
            for (int m = 0; m < NV; ++m) {
                float xv[VW];
                unpack<VW>(xr[m * kWave + lane], xv);
#pragma unroll
                for (int e = 0; e < VW; ++e) acc[e] = fmaf(uv[m][e], xv[e], acc[e]);
                if (NV > 4 && (m & 3) == 3) __builtin_amdgcn_sched_barrier(0);
            }
            return wave_sum(combine<VW>(acc));
        };
        int seg = 0;
        while (seg + 1 < a.S && a.seg_start[seg + 1] <= a.t0) ++seg;
        int64_t next_seg = seg + 1 < a.S ? a.seg_start[seg + 1] : INT64_MAX;   // absolute round
        load_u(seg);
        float z = dot_u(xrow(0)), zreg = 0.f;
        float *zrow = a.Z + (int64_t)r * a.zl.zs_r + (int64_t)K * a.zl.zs_i;
        for (int k = 0; k < ntiles; ++k) {
            if (k + 2 < ntiles) issue_tile(k + 2);
            const int rmax = min(RT, n - k * RT);
#pragma unroll 1
            for (int rr = 0; rr < rmax; ++rr) {
                const int t = k * RT + rr;
                if (lane == (t & 63)) zreg = z;
                if (a.t0 + t + 1 == next_seg) {     // the next round starts a new segment
                    ++seg;
                    next_seg = seg + 1 < a.S ? a.seg_start[seg + 1] : INT64_MAX;
                    load_u(seg);
                }
                z = dot_u(xrow(t + 1));
                if ((t & 63) == 63 || t == n - 1) {
                    const int tb = t & ~63;
                    if (tb + lane <= t) zrow[(int64_t)(tb + lane) * a.zl.zs_t] = zreg;
                }
            }
            tile_sync();
        }
        return;
    }

    // ---- learner wavefront ---------------------------------------------------------------
    auto dot_total = [](const float (&p)[VW]) {
        if constexpr (NACC == 4) return (p[0] + p[1]) + (p[2] + p[3]);
        else if constexpr (NACC == 2) return p[0] + p[1];
        else return p[0];
    };
    float wv[NV][VW];           // v = iterate / sigma
    float xa[NV][VW], xb[NV][VW];   // x_t / x_{t+1}, swapping roles every round
    float sigma = a.sigma[(int64_t)r * K + i];
    float n2 = (float)a.n2[(int64_t)r * K + i];  // ||v||^2 (kept as float64 in the state)
    const float eta = a.eta[i];
    float qv, z, zreg = 0.f, yreg = 0.f, x2reg = 0.f;   // qv = <v, x_t>, z = sigma qv
    // optimistic update: the hint is ha * x_{t-1}; hp = <w^_t, x_{t-1}>; g01 = <x_{t-1}, x_t>
    float ha = 0.f, hp = 0.f, x2prev = 0.f, g01reg = 0.f;
    if (OPT) {
        ha = a.ha[(int64_t)r * K + i];
        hp = a.hp[(int64_t)r * K + i];
        x2prev = a.x2last[a.x_shared ? 0 : r];
    }
    {
        const float *src = a.V + ((int64_t)r * K + i) * d;
        float acc[VW];
#pragma unroll
        for (int e = 0; e < VW; ++e) acc[e] = 0.f;
#pragma unroll
        for (int m = 0; m < NV; ++m) {
            unpack<VW>(xrow(0)[m * kWave + lane], xa[m]);
#pragma unroll
            for (int e = 0; e < VW; ++e) {
                const int j = (m * kWave + lane) * VW + e;
                wv[m][e] = j < d ? src[j] : 0.f;
                acc[e & (NACC - 1)] = fmaf(wv[m][e], xa[m][e], acc[e & (NACC - 1)]);   // same order as the passes
                xb[m][e] = 0.f;
            }
        }
        qv = wave_sum(dot_total(acc));
        z = sigma * qv;                               // z_0 = <w_0, x_0>
    }
    const float *x2row = a.x2 + (a.x_shared ? 0 : (int64_t)r * a.x2_run_stride);
    const float *g01row = OPT ? a.g01 + (a.x_shared ? 0 : (int64_t)r * a.x2_run_stride) : nullptr;
    const int phase = (int)(a.t0 & 63);               // exact norms at absolute rounds = 63 mod 64

    const float D = a.D;
    const float D2 = D * D;
    float *zrow = a.Z + (int64_t)r * a.zl.zs_r + (int64_t)i * a.zl.zs_i;
    // sigma changes only when a projection is active (and only downwards): its reciprocal and
    // the threshold D^2 / sigma^2 on ||v||^2 are functions of sigma alone, recomputed with it,
    // so that a round that does not project pays one compare for the projection
    float isig = fast_rcp(sigma);
    float thr = D2 * isig * isig;
    const float eta2 = 2.0f * eta;

    // the pass over the registers: step and next-round dot
    auto pass = [&](float b, const V *xr, float (&xc)[NV][VW], float (&xn)[NV][VW], float (&aq)[VW]) {
#pragma unroll
        for (int e = 0; e < VW; ++e) aq[e] = 0.f;
#pragma unroll
        for (int j = 0; j < CH; ++j) unpack<VW>(xr[j * kWave + lane], xn[j]);
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            if (c + 1 < NCH) {
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    const int m = (c + 1) * CH + j;
                    unpack<VW>(xr[m * kWave + lane], xn[m]);
                }
            }
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                const int m = c * CH + j;
#pragma unroll
                for (int e = 0; e < VW; ++e) {
                    const float w1 = fmaf(-b, xc[m][e], wv[m][e]);
                    wv[m][e] = w1;
                    aq[e & (NACC - 1)] = fmaf(w1, xn[m][e], aq[e & (NACC - 1)]);
                }
            }
            if (NCH > 2) __builtin_amdgcn_sched_barrier(0);
        }
    };

    // The same pass with one register set: chunk c of x_t is dead once the step has used it and
    // is refilled with chunk c of x_{t+1}; the dot runs kLag chunks behind so that the LDS
    // latency of the refill is covered.  Same operations in the same order as `pass`.
    auto pass_one = [&](float b, const V *xr, float (&xc)[NV][VW], float (&aq)[VW]) {
        if constexpr (kOneRowSet<NPL>) {
            static_assert(CH == 2 && VW == 4, "the ordering pin below lists the 8 values of a chunk");
            constexpr int kLag = 3;
            typedef float f4 __attribute__((ext_vector_type(4)));
            typedef const __attribute__((address_space(3))) f4 *LdsRow;
            LdsRow row = (LdsRow)(xr + lane);
#pragma unroll
            for (int e = 0; e < VW; ++e) aq[e] = 0.f;
#pragma unroll
            for (int c = 0; c < NCH + kLag; ++c) {
                if (c < NCH) {
                    const int m0 = c * CH;
#pragma unroll
                    for (int j = 0; j < CH; ++j)
#pragma unroll
                        for (int e = 0; e < VW; ++e) wv[m0 + j][e] = fmaf(-b, xc[m0 + j][e], wv[m0 + j][e]);
                    // the refill may only be issued once the step has read the old chunk: without
                    // this the LDS reads are hoisted to the top of the round (they do not depend
                    // on b) and both rows are live at once
                    asm volatile("" : "+v"(row)
                                 : "v"(wv[m0][0]), "v"(wv[m0][1]), "v"(wv[m0][2]), "v"(wv[m0][3]),
                                   "v"(wv[m0 + 1][0]), "v"(wv[m0 + 1][1]), "v"(wv[m0 + 1][2]), "v"(wv[m0 + 1][3]));
#pragma unroll
                    for (int j = 0; j < CH; ++j) {
                        const f4 fresh = row[(m0 + j) * kWave];
                        xc[m0 + j][0] = fresh.x; xc[m0 + j][1] = fresh.y;
                        xc[m0 + j][2] = fresh.z; xc[m0 + j][3] = fresh.w;
                    }
                }
                if (c >= kLag) {
#pragma unroll
                    for (int j = 0; j < CH; ++j) {
                        const int m = (c - kLag) * CH + j;
#pragma unroll
                        for (int e = 0; e < VW; ++e) aq[e & (NACC - 1)] = fmaf(wv[m][e], xc[m][e], aq[e & (NACC - 1)]);
                    }
                }
            }
        }
    };

    // Labels, ||x||^2 and <x_{t-1}, x_t> of the 64 rounds from t on, a lane each (t is a multiple of 64), and the
    // predictions of the rounds (t & ~63) .. t to Z: both happen at tile boundaries only (a tile's length divides
    // 64), so the tile loop does them and a round does not test for them.
    auto load_round_scalars = [&](int t) {
        if (yrow) yreg = (t + lane < n) ? yrow[t + lane] : 0.f;
        x2reg = (t + lane < n) ? x2row[t + lane] : 0.f;
        if (OPT) g01reg = (t + lane < n) ? g01row[t + lane] : 0.f;
    };
    auto flush_predictions = [&](int t) {
        const int tb = t & ~63;
        if (tb + lane <= t) zrow[(int64_t)(tb + lane) * a.zl.zs_t] = zreg;
    };
    // one round: consumes xc = x_t, fills xn = x_{t+1} from xnext; remeasure: ||v||^2 is summed afresh after the step
    auto round = [&](int t, const V *xnext, bool remeasure, float (&xc)[NV][VW], float (&xn)[NV][VW]) {
        const float yt = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(yreg), t & 63));
        const float x2t = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x2reg), t & 63));
        // the prediction that is played and scored: plain, z = <w_t, x_t>; optimistic,
        // w_t = s (w^_t - ha x_{t-1}) with s from ||w^_t - ha x_{t-1}||^2, all from scalars
        float zp = z;
        if (OPT) {
            const float g01t = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(g01reg), t & 63));
            // ||w^_t - ha x_{t-1}||^2 in float32 like its inputs: it only matters where it exceeds D^2,
            // and there no term is much larger than the result
            const float mf = fmaf(ha * ha, x2prev, fmaf(-2.f * ha, hp, sigma * sigma * n2));
            const float sp = mf > D2 ? D * __builtin_amdgcn_rsqf(mf) : 1.f;
            zp = sp * fmaf(-ha, g01t, z);
        }
        if (lane == (t & 63)) zreg = zp;
        // fold sigma into v first (never between computing z and using it, so that z is
        // the same whether or not a call boundary falls here)
        if (sigma < kFoldLo) {                           // (sigma never grows: no upper test)
#pragma unroll
            for (int m = 0; m < NV; ++m)
#pragma unroll
                for (int e = 0; e < VW; ++e) wv[m][e] *= sigma;
            n2 *= sigma * sigma;
            qv = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(z)));   // (uniform, like the sum it replaces)
            sigma = 1.f;
            isig = 1.f;
            thr = D2;
        }
        // w-space step along x_t; for the squared loss eta * 2 (z - y) = (2 eta) (z - y) exactly
        const float step = LOSS == 1 ? eta2 * (zp - yt) : eta * slope<LOSS>(zp, yt);
        const float b = step * isig;
        const float qold = qv;
        float aq[VW];
        if constexpr (kOneRowSet<NPL>) pass_one(b, xnext, xc, aq);
        else pass(b, xnext, xc, xn, aq);
        n2 = fmaxf(fmaf(b, fmaf(b, x2t, -2.f * qv), n2), 0.f);
        if (remeasure) {                                 // re-measure ||v||^2 exactly (replaces the identity's value)
            float an[VW];
#pragma unroll
            for (int e = 0; e < VW; ++e) an[e] = 0.f;
#pragma unroll
            for (int m = 0; m < NV; ++m)
#pragma unroll
                for (int e = 0; e < VW; ++e) an[e] = fmaf(wv[m][e], wv[m][e], an[e]);
            n2 = wave_sum(combine<VW>(an));
        }
        qv = wave_sum(dot_total(aq));                      // <v, x_{t+1}>
        const float nrm = n2;                            // ||v||^2
        if (__builtin_amdgcn_ballot_w64(nrm > thr) != 0) {   // projection (the same in every lane)
            asm volatile("" ::: "memory");    // keeps the branch: its body is not to be run speculatively
            sigma = D * __builtin_amdgcn_rsqf(nrm);
            isig = fast_rcp(sigma);
            thr = D2 * isig * isig;
        }
        z = sigma * qv;
        if (OPT) {                                       // next round's hint and <w^_{t+1}, x_t>
            hp = sigma * fmaf(-b, x2t, qold);
            ha = step;
            x2prev = x2t;
        }
    };

    static_assert(64 % RT == 0, "tiles do not straddle the 64-round groups of labels and predictions");
    for (int k = 0; k < ntiles; ++k) {
        if (k + 2 < ntiles) issue_tile(k + 2);
        const int t0 = k * RT;
        const int rmax = min(RT, n - t0);
        if ((t0 & 63) == 0) load_round_scalars(t0);
        // rows of this tile follow one another in the ring; the row after its last is the next tile's first
        const float *rows = ring + (k % kRing) * TILE, *rows_next = ring + ((k + 1) % kRing) * TILE;
        const int rm = (63 - phase - t0) & 63;               // the round of this tile (if < RT) after which ||v||^2 is re-measured
        if constexpr (kOneRowSet<NPL>) {
#pragma unroll 1
            for (int rr = 0; rr < rmax; ++rr)
                round(t0 + rr, reinterpret_cast<const V *>(rr + 1 < RT ? rows + (rr + 1) * DP : rows_next), rr == rm, xa, xa);
        } else {
#pragma unroll 1
            for (int rr = 0; rr < rmax; rr += 2) {
                const int t = t0 + rr;
                round(t, reinterpret_cast<const V *>(rows + (rr + 1) * DP), rr == rm, xa, xb);          // (RT is even)
                if (rr + 1 < rmax)
                    round(t + 1, reinterpret_cast<const V *>(rr + 2 < RT ? rows + (rr + 2) * DP : rows_next), rr + 1 == rm, xb, xa);
            }
        }
        const int tl = t0 + rmax - 1;
        if ((tl & 63) == 63 || tl == n - 1) flush_predictions(tl);
        tile_sync();   // every wavefront has drained its copies: tile k+1 is complete; tile k may be overwritten
    }

    {
        float *dst = a.V + ((int64_t)r * K + i) * d;
#pragma unroll
        for (int m = 0; m < NV; ++m)
#pragma unroll
            for (int e = 0; e < VW; ++e) {
                const int j = (m * kWave + lane) * VW + e;
                if (j < d) dst[j] = wv[m][e];
            }
        if (lane == 0) { a.sigma[(int64_t)r * K + i] = sigma; a.n2[(int64_t)r * K + i] = (double)n2; }
        if (OPT && lane == 0) { a.ha[(int64_t)r * K + i] = ha; a.hp[(int64_t)r * K + i] = hp; }
    }
}

// ---- two learners per wavefront ------------------------------------------------------------
// For d <= 1024 more than half of a round's instructions are its scalar section (slope, norm
// identity, reduction, projection), which every lane executes alike.  Here each half of a
// wavefront (32 lanes) owns one learner, so that section serves two learners at once; a lane
// keeps d/32 coordinates.  Shared round stream only; the comparators' predictions come from the
// contraction kernel, so every task is a learner.  Same arithmetic per learner as above except
// that sums run over 32 lanes.
template <int NPL> struct HalfCfg {
    static constexpr int RT = DenseCfg<NPL / 2>::RT;   // same tile bytes as the kernel above at equal d
    static constexpr int MAXW = NPL >= 32 ? 12 : 16;   // register budget
};

// Sum over the 32 lanes of each half of the wavefront (fixed order: xor-butterfly inside each row
// of 16 lanes, then row 1 += row 0 and row 3 += row 2); every lane gets the sum of its half.
__device__ __forceinline__ float half_sum(float v, bool upper)
{
    v += dpp_term<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
    v += dpp_term<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
    v += dpp_term<0x141, 0xF>(v);   // row_half_mirror
    v += dpp_term<0x140, 0xF>(v);   // row_mirror
    asm("s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 0"
        : "+v"(v));
    const float lo = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 31));
    const float hi = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
    return upper ? hi : lo;
}

template <int NPL, int LOSS, bool OPT>
__global__ void __launch_bounds__(HalfCfg<NPL>::MAXW * kWave)
dense_rounds_half_kernel(const DenseArgs a)
{
    constexpr int LW = 32;                      // lanes per learner
    constexpr int VW = 4;
    constexpr int NV = NPL / VW;
    constexpr int DP = NPL * LW;                // padded dimension
    constexpr int RT = HalfCfg<NPL>::RT;
    constexpr int TILE = RT * DP;
    constexpr int RING_ROUNDS = kRing * RT;
    constexpr int NI = TILE / 4 / kWave;
    constexpr int CH = NV >= 2 ? 2 : 1;
    constexpr int NCH = NV / CH;
    static_assert(NPL % 4 == 0 && TILE % (4 * kWave) == 0 && RT % 2 == 0, "tile shape");
    using V = float4;

    extern __shared__ float4 smem4[];
    float *ring = reinterpret_cast<float *>(smem4);

    const int tid = threadIdx.x;
    const int nthreads = blockDim.x;
    const int wpb = nthreads >> 6;
    const int lane = tid & 63;
    const int ll = lane & (LW - 1);             // lane inside the half
    const bool upper = lane >= LW;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n = a.n;
    const int d = a.d;
    const int K = a.K;

    // task = learner (run r, index i); the upper half of the last wavefront may have none: it
    // then repeats the last task and stores nothing
    const int64_t ntask = (int64_t)a.R * K;
    const int64_t q0 = 2 * ((int64_t)blockIdx.x * wpb + wave);
    const bool active = q0 < ntask;             // per wavefront
    const int64_t qraw = q0 + (upper ? 1 : 0);
    const bool store = qraw < ntask;
    const int64_t q = store ? qraw : ntask - 1;
    const int r = (int)(q / K), i = (int)(q % K);
    const float *xg = a.x;

    auto issue_tile = [&](int k) {
        float *dst = ring + (k % kRing) * TILE;
        if (a.vec_ok) {
            for (int ii = wave; ii < NI; ii += wpb) {
                const int e = ii * kWave + lane;               // float4 index in the tile
                const int rr = e / (DP / 4), j4 = e % (DP / 4);
                const int tt = k * RT + rr;
                if (tt < n && j4 * 4 < d)
                    __builtin_amdgcn_global_load_lds(
                        (const __attribute__((address_space(1))) void *)(xg + (int64_t)tt * d + j4 * 4),
                        (__attribute__((address_space(3))) void *)(dst + ii * 4 * kWave), 16, 0, 0);
            }
        } else {
            for (int e = tid; e < TILE; e += nthreads) {
                const int rr = e / DP, j = e % DP;
                const int tt = k * RT + rr;
                if (tt < n && j < d) dst[e] = xg[(int64_t)tt * d + j];
            }
        }
    };

    for (int e = tid; e < kRing * TILE / 4; e += nthreads) smem4[e] = make_float4(0.f, 0.f, 0.f, 0.f);
    tile_sync();
    const int ntiles = (n + RT - 1) / RT;
    issue_tile(0);
    if (ntiles > 1) issue_tile(1);
    tile_sync();

    auto xrow = [&](int t) { return reinterpret_cast<const V *>(ring + (t % RING_ROUNDS) * DP); };

    if (!active) {
        for (int k = 0; k < ntiles; ++k) {
            if (k + 2 < ntiles) issue_tile(k + 2);
            tile_sync();
        }
        return;
    }

    const float *yrow = a.y ? a.y + (int64_t)r * a.y_run_stride : nullptr;
    float wv[NV][VW];
    float xa[NV][VW], xb[NV][VW];
    float sigma = a.sigma[(int64_t)r * K + i];
    float n2 = (float)a.n2[(int64_t)r * K + i];
    const float eta = a.eta[i];
    float qv, z, zreg = 0.f, yreg = 0.f, x2reg = 0.f;
    float ha = 0.f, hp = 0.f, x2prev = 0.f, g01reg = 0.f;
    if (OPT) {
        ha = a.ha[(int64_t)r * K + i];
        hp = a.hp[(int64_t)r * K + i];
        x2prev = a.x2last[0];
    }
    {
        const float *src = a.V + ((int64_t)r * K + i) * d;
        float acc[2] = {0.f, 0.f};
#pragma unroll
        for (int m = 0; m < NV; ++m) {
            unpack<VW>(xrow(0)[m * LW + ll], xa[m]);
#pragma unroll
            for (int e = 0; e < VW; ++e) {
                const int j = (m * LW + ll) * VW + e;
                wv[m][e] = j < d ? src[j] : 0.f;
                acc[e & 1] = fmaf(wv[m][e], xa[m][e], acc[e & 1]);     // same order as the passes
                xb[m][e] = 0.f;
            }
        }
        qv = half_sum(acc[0] + acc[1], upper);
        z = sigma * qv;
    }
    const float *x2row = a.x2;
    const float *g01row = OPT ? a.g01 : nullptr;
    const int phase = (int)(a.t0 & 63);
    const float D = a.D;
    const float D2 = D * D;
    float *zrow = a.Z + (int64_t)r * a.zl.zs_r + (int64_t)i * a.zl.zs_i;
    float isig = fast_rcp(sigma);
    float thr = D2 * isig * isig;
    const float eta2 = 2.0f * eta;

    auto pass = [&](float b, const V *xr, float (&xc)[NV][VW], float (&xn)[NV][VW], float (&aq)[2]) {
        aq[0] = aq[1] = 0.f;
#pragma unroll
        for (int j = 0; j < CH; ++j) unpack<VW>(xr[j * LW + ll], xn[j]);
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            if (c + 1 < NCH) {
#pragma unroll
                for (int j = 0; j < CH; ++j) {
                    const int m = (c + 1) * CH + j;
                    unpack<VW>(xr[m * LW + ll], xn[m]);
                }
            }
#pragma unroll
            for (int j = 0; j < CH; ++j) {
                const int m = c * CH + j;
#pragma unroll
                for (int e = 0; e < VW; ++e) {
                    const float w1 = fmaf(-b, xc[m][e], wv[m][e]);
                    wv[m][e] = w1;
                    aq[e & 1] = fmaf(w1, xn[m][e], aq[e & 1]);
                }
            }
            if (NCH > 2) __builtin_amdgcn_sched_barrier(0);
        }
    };

    auto round = [&](int t, float (&xc)[NV][VW], float (&xn)[NV][VW]) {
        if ((t & (LW - 1)) == 0 && yrow) yreg = (t + ll < n) ? yrow[t + ll] : 0.f;   // per half: the runs may differ
        if ((t & 63) == 0) {
            x2reg = (t + lane < n) ? x2row[t + lane] : 0.f;
            if (OPT) g01reg = (t + lane < n) ? g01row[t + lane] : 0.f;
        }
        const float ylo = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(yreg), t & (LW - 1)));
        const float yhi = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(yreg), LW + (t & (LW - 1))));
        const float yt = upper ? yhi : ylo;
        const float x2t = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x2reg), t & 63));
        float zp = z;
        if (OPT) {
            const float g01t = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(g01reg), t & 63));
            // ||w^_t - ha x_{t-1}||^2 in float32 like its inputs: it only matters where it exceeds D^2,
            // and there no term is much larger than the result
            const float mf = fmaf(ha * ha, x2prev, fmaf(-2.f * ha, hp, sigma * sigma * n2));
            const float sp = mf > D2 ? D * __builtin_amdgcn_rsqf(mf) : 1.f;
            zp = sp * fmaf(-ha, g01t, z);
        }
        if (ll == (t & (LW - 1))) zreg = zp;
        if (sigma < kFoldLo) {                           // per learner: the halves may differ
#pragma unroll
            for (int m = 0; m < NV; ++m)
#pragma unroll
                for (int e = 0; e < VW; ++e) wv[m][e] *= sigma;
            n2 *= sigma * sigma;
            qv = z;
            sigma = 1.f;
            isig = 1.f;
            thr = D2;
        }
        const float step = LOSS == 1 ? eta2 * (zp - yt) : eta * slope<LOSS>(zp, yt);
        const float b = step * isig;
        const float qold = qv;
        float aq[2];
        pass(b, xrow(t + 1), xc, xn, aq);
        if (((phase + t) & 63) == 63) {                  // re-measure ||v||^2 exactly
            float an[2] = {0.f, 0.f};
#pragma unroll
            for (int m = 0; m < NV; ++m)
#pragma unroll
                for (int e = 0; e < VW; ++e) an[e & 1] = fmaf(wv[m][e], wv[m][e], an[e & 1]);
            n2 = half_sum(an[0] + an[1], upper);
        } else {
            n2 = fmaxf(fmaf(b, fmaf(b, x2t, -2.f * qv), n2), 0.f);
        }
        qv = half_sum(aq[0] + aq[1], upper);             // <v, x_{t+1}>
        const float nrm = n2;
        const bool pj = nrm > thr;                       // projection, per learner
        if (__builtin_amdgcn_ballot_w64(pj) != 0) {
            asm volatile("" ::: "memory");               // keeps the branch
            const float s2 = D * __builtin_amdgcn_rsqf(nrm);
            const float i2 = fast_rcp(s2);
            sigma = pj ? s2 : sigma;
            isig = pj ? i2 : isig;
            thr = pj ? D2 * i2 * i2 : thr;
        }
        z = sigma * qv;
        if (OPT) {
            hp = sigma * fmaf(-b, x2t, qold);
            ha = step;
            x2prev = x2t;
        }
        if ((t & (LW - 1)) == LW - 1 || t == n - 1) {    // flush the z of rounds (t & ~31) .. t
            const int tb = t & ~(LW - 1);
            if (tb + ll <= t && store) zrow[(int64_t)(tb + ll) * a.zl.zs_t] = zreg;
        }
    };

    for (int k = 0; k < ntiles; ++k) {
        if (k + 2 < ntiles) issue_tile(k + 2);
        const int rmax = min(RT, n - k * RT);
#pragma unroll 1
        for (int rr = 0; rr < rmax; rr += 2) {
            const int t = k * RT + rr;
            round(t, xa, xb);
            if (rr + 1 < rmax) round(t + 1, xb, xa);
        }
        tile_sync();
    }

    if (store) {
        float *dst = a.V + ((int64_t)r * K + i) * d;
#pragma unroll
        for (int m = 0; m < NV; ++m)
#pragma unroll
            for (int e = 0; e < VW; ++e) {
                const int j = (m * LW + ll) * VW + e;
                if (j < d) dst[j] = wv[m][e];
            }
        if (ll == 0) { a.sigma[(int64_t)r * K + i] = sigma; a.n2[(int64_t)r * K + i] = (double)n2; }
        if (OPT && ll == 0) { a.ha[(int64_t)r * K + i] = ha; a.hp[(int64_t)r * K + i] = hp; }
    }
}

// ||x_t||^2 of every round row and, if g01 is given, <x_{t-1}, x_t> (x_{-1} = the last row of the
// previous call, kept in xlast): one wavefront per row, fixed summation order.
__global__ void __launch_bounds__(256) xnorm2_kernel(const float *x, int64_t run_stride, int nruns,
                                                     int n, int d, float *out, int64_t out_stride,
                                                     float *g01, const float *xlast)
{
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= (int64_t)nruns * n) return;
    const int rr = (int)(row / n), t = (int)(row % n);
    const float *src = x + (int64_t)rr * run_stride + (int64_t)t * d;
    float acc = 0.f;
    for (int j = lane; j < d; j += 64) acc = fmaf(src[j], src[j], acc);
    const float tot = wave_sum(acc);
    if (lane == 0) out[(int64_t)rr * out_stride + t] = tot;
    if (g01) {
        const float *prev = t > 0 ? src - d : xlast + (int64_t)rr * d;
        float ac2 = 0.f;
        for (int j = lane; j < d; j += 64) ac2 = fmaf(prev[j], src[j], ac2);
        const float t2 = wave_sum(ac2);
        if (lane == 0) g01[(int64_t)rr * out_stride + t] = t2;
    }
}

// keeps the last round row of a call (and its squared norm) for the next call's hint terms
__global__ void __launch_bounds__(256) keep_last_row_kernel(const float *x, int64_t run_stride, int n, int d,
                                                            const float *x2, int64_t x2_stride, float *xlast,
                                                            float *x2last)
{
    const int rr = blockIdx.y;
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j < d) xlast[(int64_t)rr * d + j] = x[(int64_t)rr * run_stride + (int64_t)(n - 1) * d + j];
    if (j == 0) x2last[rr] = x2[(int64_t)rr * x2_stride + n - 1];
}

// Duration of one pass of the grid with l wavefronts on each SIMD, in units of a pass with one,
// fitted to sweeps on MI355X: up to about four wavefronts per SIMD mostly fill each other's
// stalls (the round is a dependent chain), beyond that they share the issue slots.
static double pass_cost(double l)
{
    return l <= 1.0 ? 1.0 : l <= 4.0 ? 1.0 + 0.1 * (l - 1.0) : l <= 6.0 ? 1.3 + 0.2 * (l - 4.0) : 1.7 + 0.55 * (l - 6.0);
}

// how one call's round kernel is launched: fixed for the call, used for each of its pieces
struct DensePlan {
    void (*kern)(const DenseArgs) = nullptr;
    size_t smem = 0;
    int wpb = 0;              // wavefronts per workgroup
    int64_t nwg = 0;          // workgroups
    int64_t batches = 0;      // passes the grid needs when the chip cannot hold it at once
    double cost = 0.0;        // modelled duration, in units of one lightly loaded pass
};

template <int NPL>
hipError_t plan_npl(const DenseArgs &a, int loss, DensePlan *plan)
{
    using C = DenseCfg<NPL>;
    const size_t smem = sizeof(float) * kRing * C::RT * NPL * kWave;
    void (*kern)(const DenseArgs) = nullptr;
    switch (loss * 2 + (a.optimistic ? 1 : 0)) {
        case 0: kern = dense_rounds_kernel<NPL, 0, false>; break;
        case 1: kern = dense_rounds_kernel<NPL, 0, true>; break;
        case 2: kern = dense_rounds_kernel<NPL, 1, false>; break;
        case 3: kern = dense_rounds_kernel<NPL, 1, true>; break;
        case 4: kern = dense_rounds_kernel<NPL, 2, false>; break;
        case 5: kern = dense_rounds_kernel<NPL, 2, true>; break;
        default: return hipErrorInvalidValue;
    }
    if (smem > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    int dev = 0, ncu = 256;
    if (hipGetDevice(&dev) == hipSuccess)
        (void)hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev);
    if (ncu <= 0) ncu = 256;

    // Wavefronts per workgroup: the value that leaves the least work on the busiest compute
    // unit.  A unit gets ceil(nWG / ncu) workgroups, c of them resident at a time: so many full
    // passes plus a last, emptier one.  A pass puts l = resident*wpb/4 wavefronts on each SIMD
    // and its duration grows with l as g(l), fitted to sweeps on MI355X: up to about four
    // wavefronts per SIMD mostly fill each other's stalls (the round is a dependent chain),
    // beyond that they share the issue slots.
    const int per_run = a.per_run;
    int best = 0;
    double best_cost = 0.0;
    for (int w = C::MAXW; w >= 1; --w) {
        // A workgroup's wavefronts are dealt to the four SIMDs in turn and there is a barrier per
        // tile, so sizes that are not a multiple of four leave SIMDs unevenly loaded (measured up
        // to 20-60 % slower at equal occupancy): they pay a penalty and win only where they save a
        // pass of the grid.  Tiny workgroups only for tiny runs.
        if (w < 3 && !(per_run < 4 && w == per_run)) continue;
        int c = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&c, reinterpret_cast<const void *>(kern),
                                                         w * kWave, smem) != hipSuccess || c <= 0)
            continue;
        const int64_t nwg = a.x_shared ? ((int64_t)a.R * per_run + w - 1) / w
                                       : (int64_t)a.R * ((per_run + w - 1) / w);
        const int64_t per_cu = (nwg + ncu - 1) / ncu;
        const int64_t full = per_cu / c, rem = per_cu % c;
        double cost = (double)full * pass_cost((double)(c * w) / 4.0) + (rem ? pass_cost((double)(rem * w) / 4.0) : 0.0);
        if (w % 4 != 0 && per_run % w != 0) cost *= 1.1;
        // on equal cost prefer more, smaller workgroups per unit (fewer wavefronts held up by one
        // barrier), down to eight wavefronts (below that the per-workgroup staging of x shows)
        const bool better = best == 0 || cost < best_cost * (1.0 - 1e-9) ||
                            (w >= 8 && cost <= best_cost * (1.0 + 1e-9));
        if (better) { best = w; best_cost = cost; }
    }
    {                                                     // tuning choice: wavefronts per workgroup
        const int w = (int)a.tune->get(OCO_OPT_DENSE_WPB);
        if (w >= 1 && w <= C::MAXW) best = w;
    }
    if (best == 0) return hipErrorInvalidConfiguration;
    plan->cost = best_cost;
    if (a.tune->get(OCO_OPT_VERBOSE) == 1)
        fprintf(stderr, "dense plan: NPL %d per_run %d -> wpb %d cost %.3f\n", NPL, per_run, best, best_cost);
    int c = 1;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&c, reinterpret_cast<const void *>(kern), best * kWave,
                                                     smem) != hipSuccess || c <= 0)
        c = 1;
    plan->kern = kern;
    plan->smem = smem;
    plan->wpb = best;
    plan->nwg = a.x_shared ? ((int64_t)a.R * per_run + best - 1) / best
                           : (int64_t)a.R * ((per_run + best - 1) / best);
    plan->batches = ((plan->nwg + ncu - 1) / ncu + c - 1) / c;
    return hipSuccess;
}

// the same for the kernel with two learners per wavefront (shared stream, learners only)
template <int NPL>
hipError_t plan_half(const DenseArgs &a, int loss, DensePlan *plan)
{
    using C = HalfCfg<NPL>;
    const size_t smem = sizeof(float) * kRing * C::RT * NPL * 32;
    void (*kern)(const DenseArgs) = nullptr;
    switch (loss * 2 + (a.optimistic ? 1 : 0)) {
        case 0: kern = dense_rounds_half_kernel<NPL, 0, false>; break;
        case 1: kern = dense_rounds_half_kernel<NPL, 0, true>; break;
        case 2: kern = dense_rounds_half_kernel<NPL, 1, false>; break;
        case 3: kern = dense_rounds_half_kernel<NPL, 1, true>; break;
        case 4: kern = dense_rounds_half_kernel<NPL, 2, false>; break;
        case 5: kern = dense_rounds_half_kernel<NPL, 2, true>; break;
        default: return hipErrorInvalidValue;
    }
    if (smem > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    int dev = 0, ncu = 256;
    if (hipGetDevice(&dev) == hipSuccess)
        (void)hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev);
    if (ncu <= 0) ncu = 256;
    const int64_t nwaves = ((int64_t)a.R * a.K + 1) / 2;
    int best = 0, best_c = 1;
    double best_cost = 0.0;
    for (int w = C::MAXW; w >= 3; --w) {
        int c = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&c, reinterpret_cast<const void *>(kern),
                                                         w * kWave, smem) != hipSuccess || c <= 0)
            continue;
        const int64_t nwg = (nwaves + w - 1) / w;
        const int64_t per_cu = (nwg + ncu - 1) / ncu;
        const int64_t full = per_cu / c, rem = per_cu % c;
        double cost = (double)full * pass_cost((double)(c * w) / 4.0) + (rem ? pass_cost((double)(rem * w) / 4.0) : 0.0);
        if (w % 4 != 0) cost *= 1.1;
        const bool better = best == 0 || cost < best_cost * (1.0 - 1e-9) || (w >= 8 && cost <= best_cost * (1.0 + 1e-9));
        if (better) { best = w; best_cost = cost; best_c = c; }
    }
    {                                                     // tuning choice
        const int w = (int)a.tune->get(OCO_OPT_DENSE_WPB);
        if (w >= 1 && w <= C::MAXW) best = w;
    }
    if (best == 0) return hipErrorInvalidConfiguration;
    plan->kern = kern;
    plan->smem = smem;
    plan->wpb = best;
    plan->nwg = (nwaves + best - 1) / best;
    plan->batches = ((plan->nwg + ncu - 1) / ncu + best_c - 1) / best_c;
    plan->cost = best_cost;
    if (a.tune->get(OCO_OPT_VERBOSE) == 1)
        fprintf(stderr, "dense plan (two learners per wavefront): NPL %d -> wpb %d cost %.3f\n", NPL, best, best_cost);
    return hipSuccess;
}

hipError_t launch_piece(const DensePlan &p, const DenseArgs &a, hipStream_t s)
{
    const int per_run = a.per_run;
    dim3 grid;
    if (a.x_shared)
        grid = dim3((unsigned)p.nwg, 1, 1);
    else
        grid = dim3((unsigned)((per_run + p.wpb - 1) / p.wpb), (unsigned)a.R, 1);
    hipError_t e = clock_begin(a.clock, s, "dense_round_kernel");
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(p.kern, grid, dim3(p.wpb * kWave), p.smem, s, a);
    e = hipGetLastError();
    return e != hipSuccess ? e : clock_end(a.clock, s);
}

}  // namespace

bool dense_supported(int64_t d, int x_shared) { return d >= 1 && d <= (x_shared ? OCO_MAX_DENSE_D : 64 * kWave); }

// The scalars of the round rows that the hint terms of the optimistic update need, for the rounds of a.n
// (all runs): ||x_t||^2 into a.x2 and <x_{t-1}, x_t> into a.g01 (x_{-1}: the row kept from the call before).
hipError_t launch_hint_scalars(const DenseArgs &a, hipStream_t s)
{
    const int nruns = a.x_shared ? 1 : a.R;
    const int64_t xstride = a.x_shared ? 0 : a.x_run_stride;
    const int64_t rows = (int64_t)nruns * a.n;
    hipLaunchKernelGGL(xnorm2_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, a.x, xstride, nruns,
                       a.n, a.d, a.x2, a.x2_run_stride, a.g01, a.xlast);
    return hipGetLastError();
}

// ... and the last row of the call with its squared norm, kept for the next call (a.x2 filled as above)
hipError_t launch_keep_last_row(const DenseArgs &a, hipStream_t s)
{
    const int nruns = a.x_shared ? 1 : a.R;
    const int64_t xstride = a.x_shared ? 0 : a.x_run_stride;
    hipLaunchKernelGGL(keep_last_row_kernel, dim3((unsigned)((a.d + 255) / 256), (unsigned)nruns), dim3(256), 0, s,
                       a.x, xstride, a.n, a.d, a.x2, a.x2_run_stride, a.xlast, a.x2last);
    return hipGetLastError();
}

// One piece of a call: the squared norms of its rows, its round kernel, and the row kept for the
// next piece's hint terms.
static hipError_t launch_dense_piece(const DensePlan &plan, const DenseArgs &a, hipStream_t s)
{
    const int nruns = a.x_shared ? 1 : a.R;
    const int64_t xstride = a.x_shared ? 0 : a.x_run_stride;
    const int64_t rows = (int64_t)nruns * a.n;
    hipLaunchKernelGGL(xnorm2_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, a.x, xstride, nruns,
                       a.n, a.d, a.x2, a.x2_run_stride, a.optimistic ? a.g01 : nullptr,
                       a.optimistic ? a.xlast : nullptr);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (a.per_run == a.K) {
        ComparatorGemmArgs g{};
        g.x = a.x; g.u = a.u; g.seg_start = a.seg_start; g.S = a.S; g.Z = a.Z; g.zl = a.zl;
        g.d = a.d; g.K = a.K; g.R = a.R; g.t0 = a.t0; g.n = a.n; g.vec_ok = a.vec_ok;
        e = launch_comparator_gemm(g, s);
        if (e != hipSuccess) return e;
    }
    e = launch_piece(plan, a, s);
    if (e != hipSuccess || !a.optimistic) return e;
    hipLaunchKernelGGL(keep_last_row_kernel, dim3((unsigned)((a.d + 255) / 256), (unsigned)nruns), dim3(256), 0, s,
                       a.x, xstride, a.n, a.d, a.x2, a.x2_run_stride, a.xlast, a.x2last);
    return hipGetLastError();
}

// Works out how the round kernel of this configuration is launched (kernel, workgroup size,
// who takes the comparators' predictions).
static hipError_t make_dense_plan(DenseArgs &a, int loss, DensePlan *out)
{
    const int npl = (a.d + kWave - 1) / kWave;
    auto make_plan = [&](DensePlan *plan) {
        if (npl <= 1) return plan_npl<1>(a, loss, plan);
        if (npl <= 2) return plan_npl<2>(a, loss, plan);
        if (npl <= 4) return plan_npl<4>(a, loss, plan);
        if (npl <= 8) return plan_npl<8>(a, loss, plan);
        if (npl <= 16) return plan_npl<16>(a, loss, plan);
        if (npl <= 32) return plan_npl<32>(a, loss, plan);
        if (npl <= 64) return plan_npl<64>(a, loss, plan);
        return hipErrorInvalidValue;
    };
    // Each run has one more wavefront task than learners, the comparator's, which only takes
    // inner products.  With a shared stream those are one contraction (U X^T per comparator
    // segment) that a kernel of its own does on the matrix cores: worth it where the round
    // kernel's grid gets cheaper without the extra tasks (fewer passes over the chip).
    DensePlan plan;
    a.per_run = a.K + 1;
    hipError_t e = make_plan(&plan);
    if (e != hipSuccess) return e;
    if (a.x_shared) {
        const int mode = (int)a.tune->get(OCO_OPT_COMPARATOR_GEMM);     // 0 never, 1 always
        DensePlan alt;
        a.per_run = a.K;
        e = make_plan(&alt);
        if (e != hipSuccess) return e;
        if (mode == 1 || (mode != 0 && alt.cost < plan.cost * 0.98)) plan = alt;
        else a.per_run = a.K + 1;
    }

    // Two learners per wavefront where a round is mostly its scalar section (d <= 1024) and the
    // grid is large enough to be bound by instruction issue rather than by the latency of a round.
    {
        bool half = a.x_shared && a.d > 96 && a.d <= 1024 && (int64_t)a.R * a.K >= kHalfMinTasks;
        const int hv = (int)a.tune->get(OCO_OPT_DENSE_HALF);          // 0 never, 1 wherever it can run
        if (hv >= 0) half = hv != 0 && a.x_shared && a.d <= 1024;
        if (half) {
            const int nplh = (a.d + 31) / 32;
            a.per_run = a.K;                                // comparators: contraction kernel
            if (nplh <= 4) e = plan_half<4>(a, loss, &plan);
            else if (nplh <= 8) e = plan_half<8>(a, loss, &plan);
            else if (nplh <= 16) e = plan_half<16>(a, loss, &plan);
            else e = plan_half<32>(a, loss, &plan);
            if (e != hipSuccess) return e;
        }
    }
    *out = plan;
    return hipSuccess;
}

hipError_t launch_dense_rounds(const DenseArgs &a0, int loss, hipStream_t s, const PieceHook *hook)
{
    if (a0.n <= 0) return hipSuccess;
    if (dense_window_wanted(a0)) return launch_dense_window(a0, loss, s, hook);
    if (a0.d > 64 * kWave) return hipErrorInvalidValue;
    DenseArgs a = a0;
    // the plan depends on the configuration and the tuning choices only: made once per state
    DensePlan plan;
    if (a.plan->valid) {
        plan.kern = reinterpret_cast<void (*)(const DenseArgs)>(const_cast<void *>(a.plan->kern));
        plan.smem = a.plan->smem; plan.wpb = a.plan->wpb; plan.nwg = a.plan->nwg;
        plan.batches = a.plan->batches;
        a.per_run = a.plan->per_run;
    } else {
        hipError_t e = make_dense_plan(a, loss, &plan);
        if (e != hipSuccess) return e;
        a.plan->kern = reinterpret_cast<const void *>(plan.kern);
        a.plan->smem = plan.smem; a.plan->wpb = plan.wpb; a.plan->nwg = plan.nwg;
        a.plan->batches = plan.batches; a.plan->per_run = a.per_run;
        a.plan->valid = true;
    }
    hipError_t e = hipSuccess;

    // Rounds give the same bits under any split of a call, so a call may go as several launches:
    //  - A grid that takes several passes over the chip has workgroups at unrelated positions of a
    //    shared round stream, whose footprint is then the whole stream: pieces of at most
    //    kStreamPieceBytes keep the stream of a piece in the last-level cache for every pass.
    //  - A grid that leaves most of the chip idle lets the caller's per-piece work (the hook) run
    //    beside the following pieces.
    int64_t pieces = 1;
    bool beside = false;
    if (plan.batches > 1 && a.x_shared) {
        const int64_t bytes = (int64_t)a.n * a.d * (int64_t)sizeof(float);
        pieces = (bytes + kStreamPieceBytes - 1) / kStreamPieceBytes;
    } else if (hook && plan.nwg * plan.wpb <= kBesideMaxWaves) {
        pieces = kBesidePieces;
        beside = true;
    }
    if (a.tune->get(OCO_OPT_DENSE_PIECES) >= 1) pieces = a.tune->get(OCO_OPT_DENSE_PIECES);   // tuning choice
    pieces = std::max<int64_t>(1, std::min<int64_t>(pieces, a.n / kPieceMinRounds));
    const int64_t step = (a.n / pieces + 63) / 64 * 64;
    for (int64_t off = 0; off < a.n; off += step) {
        const int64_t len = std::min<int64_t>(step, a.n - off);
        DenseArgs b = a;
        b.x = a.x + off * a.d; b.t0 = a.t0 + off; b.n = (int)len;
        if (b.y) b.y = a.y + off;
        b.x2 = a.x2 + off;
        if (b.g01) b.g01 = a.g01 + off;
        b.Z = a.Z + off * a.zl.zs_t;
        e = launch_dense_piece(plan, b, s);
        if (e == hipSuccess && beside) e = hook->fn(hook->ctx, (int)off, (int)len);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace oco
