// Dense rounds of the base learners (Sec. 3.1 update inside the ensemble of
// Sec. 3.3), many rounds per launch.
//
// Mapping.  One wavefront owns one base learner of one run for the whole call:
// lane l keeps d/64 coordinates of the iterate in registers, so the inner
// product <w_t^i, x_t> and the norm of the stepped vector are wavefront
// reductions (DPP) and no learner ever waits for another -- each base learner
// steps along the gradient at its own iterate.  One extra wavefront per run
// carries the comparator u_t and only takes inner products.  The wavefronts of
// a workgroup share the round stream: x is staged through LDS in tiles of RT
// rounds, double buffered, one barrier per tile.
//
// One pass over the registers per round.  The iterate is kept as w = sigma*v
// with a per-learner scalar sigma, so the projection onto the ball only
// changes sigma.  In round t the pass computes
//     v      <- v - (eta c_t / sigma) x_t          (gradient step, c_t = phi'(z_t; y_t))
//     nrm    =  ||v||^2                            (for the projection)
//     q      =  <v, x_{t+1}>                       (next round's prediction)
// then sigma <- D/||v|| if sigma ||v|| > D, and z_{t+1} = sigma q.  x_{t+1} is
// read from LDS during the pass and stays in registers as the next round's x_t.
// sigma is folded back into v, at the start of a round, once it has left
// [2^-24, 2^24].
//
// The kernel writes z_t^i for every round to Z; losses, Hedge weights and
// regret are computed from Z by the meta kernel.
#include "oco_internal.h"

namespace oco {
namespace {

template <int NPL> struct DenseCfg;
// NPL: coordinates per lane.  WPB: wavefronts per workgroup.  RT: rounds per LDS tile.
template <> struct DenseCfg<1>  { static constexpr int WPB = 4,  RT = 63; };
template <> struct DenseCfg<2>  { static constexpr int WPB = 16, RT = 31; };
template <> struct DenseCfg<4>  { static constexpr int WPB = 8,  RT = 31; };
template <> struct DenseCfg<8>  { static constexpr int WPB = 8,  RT = 15; };
template <> struct DenseCfg<16> { static constexpr int WPB = 8,  RT = 7; };
template <> struct DenseCfg<32> { static constexpr int WPB = 8,  RT = 3; };
template <> struct DenseCfg<64> { static constexpr int WPB = 8,  RT = 2; };

template <int VW> struct VecT;
template <> struct VecT<1> { using type = float; };
template <> struct VecT<2> { using type = float2; };
template <> struct VecT<4> { using type = float4; };

__device__ __forceinline__ float dpp_add(float v, const int ctrl_tag);

// Sum over the 64 lanes, result broadcast to the whole wavefront.  Fixed
// order: xor-butterfly inside each row of 16 lanes, then rows 0+1 and 2+3,
// then the two halves.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_term(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}

__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_term<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
    v += dpp_term<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
    v += dpp_term<0x141, 0xF>(v);   // row_half_mirror
    v += dpp_term<0x140, 0xF>(v);   // row_mirror
    v += dpp_term<0x142, 0xA>(v);   // row_bcast15 into rows 1 and 3
    v += dpp_term<0x143, 0xC>(v);   // row_bcast31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

template <int LOSS> __device__ __forceinline__ float slope(float z, float y)
{
    if (LOSS == 0) return 1.0f;
    if (LOSS == 1) return 2.0f * (z - y);
    // logistic: -y / (1 + exp(y z)); exp overflow gives -y/inf = 0
    return -y / (1.0f + expf(y * z));
}

template <int VW> __device__ __forceinline__ float combine(const float (&acc)[VW])
{
    if (VW == 4) return (acc[0] + acc[1]) + (acc[2] + acc[3]);
    if (VW == 2) return acc[0] + acc[1];
    return acc[0];
}

template <int NPL, int LOSS>
__global__ void __launch_bounds__(DenseCfg<NPL>::WPB * kWave)
dense_rounds_kernel(const DenseArgs a)
{
    using C = DenseCfg<NPL>;
    constexpr int VW = NPL >= 4 ? 4 : NPL;      // floats per LDS read
    constexpr int NV = NPL / VW;                // LDS reads per lane and round
    constexpr int DP = NPL * kWave;             // padded dimension
    constexpr int RT = C::RT;
    constexpr int NT = C::WPB * kWave;
    constexpr int TILE = (RT + 1) * DP;         // floats per LDS buffer (one look-ahead round)
    constexpr int TILE4 = TILE / 4;
    constexpr int PF = (TILE4 + NT - 1) / NT;   // float4 prefetch registers per thread
    using V = typename VecT<VW>::type;

    extern __shared__ float4 smem4[];
    float *xs = reinterpret_cast<float *>(smem4);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int n = a.n;
    const int d = a.d;
    const int K = a.K;

    // which (run, learner) this wavefront owns; learner K is the comparator
    int r, i;
    bool active;
    if (a.x_shared) {
        const int64_t q = (int64_t)blockIdx.x * C::WPB + wave;
        active = q < (int64_t)a.R * (K + 1);
        r = active ? (int)(q / (K + 1)) : 0;
        i = active ? (int)(q % (K + 1)) : 0;
    } else {
        r = blockIdx.y;
        i = blockIdx.x * C::WPB + wave;
        active = i <= K;
        if (!active) i = 0;
    }
    const float *xg = a.x_shared ? a.x : a.x + (int64_t)blockIdx.y * a.x_run_stride;

    // ---- cooperative staging of x: tile k holds rounds k*RT .. k*RT+RT -----
    float4 pf[PF];
    auto issue = [&](int k) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int e = p * NT + tid;
            const int rr = e / (DP / 4), j4 = e % (DP / 4);
            const int tt = k * RT + rr;
            const bool ok = e < TILE4 && tt < n && j4 * 4 < d;
            pf[p] = ok ? reinterpret_cast<const float4 *>(xg + (int64_t)tt * d)[j4]
                       : make_float4(0.f, 0.f, 0.f, 0.f);
        }
    };
    auto commit = [&](int buf) {
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            const int e = p * NT + tid;
            if (e < TILE4) reinterpret_cast<float4 *>(xs + buf * TILE)[e] = pf[p];
        }
    };
    auto stage_scalar = [&](int k, int buf) {   // any d, any alignment
        for (int e = tid; e < TILE; e += NT) {
            const int rr = e / DP, j = e % DP;
            const int tt = k * RT + rr;
            xs[buf * TILE + e] = (tt < n && j < d) ? xg[(int64_t)tt * d + j] : 0.f;
        }
    };

    const int ntiles = (n + RT - 1) / RT;
    if (a.vec_ok) { issue(0); commit(0); } else { stage_scalar(0, 0); }
    __syncthreads();

    // ---- per-wavefront state -------------------------------------------------
    float wv[NV][VW];      // v: iterate / sigma (or the comparator)
    float xc[NV][VW];      // x_t of the current round
    float sigma = 1.f, eta = 0.f, z = 0.f;
    float zreg = 0.f, yreg = 0.f;
    const bool is_cmp = (i == K);
    int seg = 0;
    int64_t next_seg = INT64_MAX;     // absolute round at which the comparator changes
    float *zrow = a.Z + (int64_t)r * a.zl.zs_r + (int64_t)i * a.zl.zs_i;
    const float *yrow = a.y ? a.y + (int64_t)r * a.y_run_stride : nullptr;

    auto load_vec = [&](const float *src) {     // src: d floats in global memory
#pragma unroll
        for (int m = 0; m < NV; ++m)
#pragma unroll
            for (int e = 0; e < VW; ++e) {
                const int j = (m * kWave + lane) * VW + e;
                wv[m][e] = j < d ? src[j] : 0.f;
            }
    };
    auto read_x = [&](const float *row, float (&dst)[NV][VW]) {
#pragma unroll
        for (int m = 0; m < NV; ++m) {
            const V t = reinterpret_cast<const V *>(row)[m * kWave + lane];
            if constexpr (VW == 4) { dst[m][0] = t.x; dst[m][1] = t.y; dst[m][2] = t.z; dst[m][3] = t.w; }
            else if constexpr (VW == 2) { dst[m][0] = t.x; dst[m][1] = t.y; }
            else { dst[m][0] = t; }
        }
    };
    auto dot_xc = [&]() {
        float acc[VW];
#pragma unroll
        for (int e = 0; e < VW; ++e) acc[e] = 0.f;
#pragma unroll
        for (int m = 0; m < NV; ++m)
#pragma unroll
            for (int e = 0; e < VW; ++e) acc[e] = fmaf(wv[m][e], xc[m][e], acc[e]);
        return wave_sum(combine<VW>(acc));
    };

    if (active) {
        if (is_cmp) {
            while (seg + 1 < a.S && a.seg_start[seg + 1] <= a.t0) ++seg;
            next_seg = seg + 1 < a.S ? a.seg_start[seg + 1] : INT64_MAX;
            load_vec(a.u + ((int64_t)r * a.S + seg) * d);
        } else {
            load_vec(a.V + ((int64_t)r * K + i) * d);
            sigma = a.sigma[(int64_t)r * K + i];
            eta = a.eta[i];
        }
        read_x(xs, xc);                 // x_0
        z = sigma * dot_xc();           // z_0 = <w_0, x_0>
    }

    const float D = a.D;
    const float D2 = D * D;

    for (int k = 0; k < ntiles; ++k) {
        const bool more = k + 1 < ntiles;
        if (more && a.vec_ok) issue(k + 1);
        const float *tile = xs + (k & 1) * TILE;
        if (active) {
            for (int rr = 0; rr < RT; ++rr) {
                const int t = k * RT + rr;
                if (t >= n) break;
                if ((t & 63) == 0 && yrow) yreg = (t + lane < n) ? yrow[t + lane] : 0.f;
                // record z_t
                if (lane == (t & 63)) zreg = z;
                const float *xnext = tile + (rr + 1) * DP;
                if (is_cmp) {
                    // comparator: no step; switch segment when the next round starts one
                    if (a.t0 + t + 1 == next_seg) {
                        ++seg;
                        next_seg = seg + 1 < a.S ? a.seg_start[seg + 1] : INT64_MAX;
                        load_vec(a.u + ((int64_t)r * a.S + seg) * d);
                    }
                    read_x(xnext, xc);
                    z = dot_xc();
                } else {
                    // fold sigma into v first (never between computing z and using it, so
                    // that z is the same whether or not a call boundary falls here)
                    if (sigma < kFoldLo || sigma > kFoldHi) {
#pragma unroll
                        for (int m = 0; m < NV; ++m)
#pragma unroll
                            for (int e = 0; e < VW; ++e) wv[m][e] *= sigma;
                        sigma = 1.f;
                    }
                    const float yt = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(yreg), t & 63));
                    const float c = slope<LOSS>(z, yt);
                    const float b = (eta * c) / sigma;
                    float an[VW], aq[VW];
#pragma unroll
                    for (int e = 0; e < VW; ++e) { an[e] = 0.f; aq[e] = 0.f; }
#pragma unroll
                    for (int m = 0; m < NV; ++m) {
                        const V xn = reinterpret_cast<const V *>(xnext)[m * kWave + lane];
                        float xnv[VW];
                        if constexpr (VW == 4) { xnv[0] = xn.x; xnv[1] = xn.y; xnv[2] = xn.z; xnv[3] = xn.w; }
                        else if constexpr (VW == 2) { xnv[0] = xn.x; xnv[1] = xn.y; }
                        else { xnv[0] = xn; }
#pragma unroll
                        for (int e = 0; e < VW; ++e) {
                            const float w1 = fmaf(-b, xc[m][e], wv[m][e]);
                            wv[m][e] = w1;
                            an[e] = fmaf(w1, w1, an[e]);
                            aq[e] = fmaf(w1, xnv[e], aq[e]);
                            xc[m][e] = xnv[e];
                        }
                    }
                    const float nrm = wave_sum(combine<VW>(an));   // ||v||^2
                    const float q = wave_sum(combine<VW>(aq));     // <v, x_{t+1}>
                    if (sigma * sigma * nrm > D2) sigma = D / sqrtf(nrm);   // projection
                    z = sigma * q;
                }
                if ((t & 63) == 63 || t == n - 1) {
                    const int tb = t & ~63;
                    if (tb + lane <= t) zrow[(int64_t)(tb + lane) * a.zl.zs_t] = zreg;
                }
            }
        }
        if (more) {
            if (a.vec_ok) commit((k + 1) & 1); else stage_scalar(k + 1, (k + 1) & 1);
        }
        __syncthreads();
    }

    if (active && !is_cmp) {
        float *dst = a.V + ((int64_t)r * K + i) * d;
#pragma unroll
        for (int m = 0; m < NV; ++m)
#pragma unroll
            for (int e = 0; e < VW; ++e) {
                const int j = (m * kWave + lane) * VW + e;
                if (j < d) dst[j] = wv[m][e];
            }
        if (lane == 0) a.sigma[(int64_t)r * K + i] = sigma;
    }
}

template <int NPL>
hipError_t launch_npl(const DenseArgs &a, int loss, hipStream_t s)
{
    using C = DenseCfg<NPL>;
    const size_t smem = sizeof(float) * 2 * (C::RT + 1) * NPL * kWave;
    dim3 grid;
    if (a.x_shared) {
        const int64_t tasks = (int64_t)a.R * (a.K + 1);
        grid = dim3((unsigned)((tasks + C::WPB - 1) / C::WPB), 1, 1);
    } else {
        grid = dim3((unsigned)((a.K + 1 + C::WPB - 1) / C::WPB), (unsigned)a.R, 1);
    }
    const dim3 block(C::WPB * kWave);
    void (*kern)(const DenseArgs) = nullptr;
    switch (loss) {
        case 0: kern = dense_rounds_kernel<NPL, 0>; break;
        case 1: kern = dense_rounds_kernel<NPL, 1>; break;
        case 2: kern = dense_rounds_kernel<NPL, 2>; break;
        default: return hipErrorInvalidValue;
    }
    if (smem > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, grid, block, smem, s, a);
    return hipGetLastError();
}

}  // namespace

bool dense_supported(int64_t d) { return d >= 1 && d <= 64 * kWave; }

hipError_t launch_dense_rounds(const DenseArgs &a, int loss, hipStream_t s)
{
    if (a.n <= 0) return hipSuccess;
    const int npl = (a.d + kWave - 1) / kWave;
    if (npl <= 1) return launch_npl<1>(a, loss, s);
    if (npl <= 2) return launch_npl<2>(a, loss, s);
    if (npl <= 4) return launch_npl<4>(a, loss, s);
    if (npl <= 8) return launch_npl<8>(a, loss, s);
    if (npl <= 16) return launch_npl<16>(a, loss, s);
    if (npl <= 32) return launch_npl<32>(a, loss, s);
    if (npl <= 64) return launch_npl<64>(a, loss, s);
    return hipErrorInvalidValue;
}

}  // namespace oco
