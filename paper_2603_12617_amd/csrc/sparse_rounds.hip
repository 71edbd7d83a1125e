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
// with the R*K learners interleaved, V[j][q], q = r*K + i: the 64 lanes of a
// wavefront are 64 learners, one coordinate of all of them is one contiguous
// 256-byte row segment, every gather and scatter is fully coalesced and all
// the per-learner scalar work (slope, step, norm, projection) runs
// lane-parallel with no reduction.
//
// The path is a dependent chain of T rounds per learner, so what matters is
// the latency of one round.  A workgroup is two wavefronts: the first runs the
// rounds; the second only reads, a bounded number of rounds ahead, one word of
// every 128-byte line the first will need, so that the gathers hit in L2
// instead of waiting for HBM.  Column indices and values of a round are one
// vector load (lane j holds entry j) issued two rounds early and broadcast
// with v_readlane.
//
// The comparator's predictions <u_t, x_t> do not depend on the learners and
// are taken by a separate, fully parallel kernel (one thread per run-round).
//
// On the boundary of the ball sigma shrinks geometrically (every projection
// multiplies it by a factor < 1) and v grows, so sigma has to be folded back
// into v now and then: V[:, q] *= sigma_q, ||v||^2 *= sigma_q^2, sigma_q = 1.
// The rounds are launched in segments that end at every 2048th round of the
// horizon; after each segment a grid-wide kernel folds the 64-learner column
// groups whose smallest sigma has dropped below 2^-20 (a streaming pass at HBM
// speed, and a no-op otherwise).  Should a sigma fall below 2^-60 inside a
// segment (steps many orders of magnitude larger than the ball), the working
// wavefront folds its own columns in place, slowly but safely.  All fold
// decisions depend on the state and the absolute round index only, so results
// do not depend on how the horizon is cut into calls.
#include "oco_internal.h"

#include <cstdlib>

namespace oco {
namespace {

template <int LOSS> __device__ __forceinline__ float slope(float z, float y)
{
    if (LOSS == 0) return 1.0f;
    if (LOSS == 1) return 2.0f * (z - y);
    return -y * __builtin_amdgcn_rcpf(1.0f + __expf(y * z));
}

constexpr double kSparseFoldLo = 0x1p-60;    // in-kernel emergency fold
constexpr double kSparseFoldSoft = 0x1p-20;  // fold between segments
constexpr int kSegment = 2048;               // rounds per launch segment (absolute alignment)
constexpr int kPrefetchAhead = 48;   // rounds the reading wavefront may run ahead
constexpr int kPrefetchBatch = 16;   // rounds whose lines it requests before waiting

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_term(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}

__device__ __forceinline__ float wave_sum(float v)     // fixed order, result uniform
{
    v += dpp_term<0xB1, 0xF>(v);
    v += dpp_term<0x4E, 0xF>(v);
    v += dpp_term<0x141, 0xF>(v);
    v += dpp_term<0x140, 0xF>(v);
    v += dpp_term<0x142, 0xA>(v);
    v += dpp_term<0x143, 0xC>(v);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

// NZ: compile-time bound on the entries per round (nnz <= NZ <= 64)
template <int NZ, int LOSS>
__global__ void __launch_bounds__(2 * kWave) sparse_rounds_kernel(const SparseArgs a)
{
    __shared__ int progress;                 // rounds finished by the first wavefront
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nnz = a.nnz;
    const int n = a.n;
    const int q0 = blockIdx.x * kWave;       // first learner (column) of this workgroup
    if (threadIdx.x == 0) progress = 0;
    __syncthreads();

    if (wave == 1) {
        if (!a.prefetch) return;
        // ---- reading wavefront: pull the lines of coming rounds into L2 ---------------
        const int j = lane & 31, half = lane >> 5;      // entry j (and j+32), first/second line
        const float *base = a.V + q0 + half * 32;
        float sink = 0.f;
        for (int tb = 0; tb < n; tb += kPrefetchBatch) {
            int spins = 0;
            while (tb > *(volatile int *)&progress + kPrefetchAhead && ++spins < (1 << 18))
                __builtin_amdgcn_s_sleep(4);
            float got[kPrefetchBatch][2];
#pragma unroll
            for (int u = 0; u < kPrefetchBatch; ++u) {
                const int t = tb + u;
                got[u][0] = got[u][1] = 0.f;
                if (t < n) {
                    if (j < nnz) got[u][0] = base[(int64_t)a.col[(int64_t)t * nnz + j] * a.RKp];
                    if (NZ > 32 && j + 32 < nnz)
                        got[u][1] = base[(int64_t)a.col[(int64_t)t * nnz + j + 32] * a.RKp];
                }
            }
#pragma unroll
            for (int u = 0; u < kPrefetchBatch; ++u) sink += got[u][0] + got[u][1];
        }
        if (sink == 1.2345e30f) a.Z[0] = sink;          // never true; keeps the loads alive
        return;
    }

    // ---- working wavefront: lane = learner q = r*K + i -------------------------------------
    const int nq = a.R * a.K;
    const int q = q0 + lane;
    const bool valid = q < nq;
    const int qq = valid ? q : 0;
    const int r = qq / a.K, i = qq % a.K;
    const float eta = valid ? a.eta[i] : 0.f;
    double sigma = a.sigma[q];
    double n2 = a.n2[q];
    const double D2 = a.D * a.D;
    float *Vq = a.V + q;                             // column of this lane (padded columns exist)
    const float *yrow = a.y ? a.y + (int64_t)r * a.y_run_stride : nullptr;
    float *zrow = a.Z + (int64_t)r * a.zl.zs_r + (int64_t)i * a.zl.zs_i;

    // entries of a round, lane j = entry j; lanes >= nnz repeat entry 0 with value 0
    const int jl = lane < nnz ? lane : 0;
    auto load_round = [&](int t, int &c, float &x, float &y) {
        if (t < n) {
            c = a.col[(int64_t)t * nnz + jl];
            x = lane < nnz ? a.val[(int64_t)t * nnz + lane] : 0.f;
            y = yrow ? yrow[t] : 0.f;
        } else { c = 0; x = 0.f; y = 0.f; }
    };
    int c0, c1, c2;
    float x0, x1, x2, y0, y1, y2;
    load_round(0, c0, x0, y0);
    load_round(1, c1, x1, y1);

    for (int t = 0; t < n; ++t) {
        // gather the touched coordinates of all 64 learners: NZ coalesced row reads
        float v[NZ], xv[NZ];
        int64_t off[NZ];
#pragma unroll
        for (int j = 0; j < NZ; ++j) {
            off[j] = (int64_t)__builtin_amdgcn_readlane(c0, j) * a.RKp;
            xv[j] = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x0), j));
            v[j] = Vq[off[j]];
        }
        load_round(t + 2, c2, x2, y2);                 // stream, two rounds early
        const float X2 = wave_sum(x0 * x0);            // ||x_t||^2 (lanes >= nnz hold 0)

        float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < NZ; ++j) acc[j & 3] = fmaf(v[j], xv[j], acc[j & 3]);
        const float qv = (acc[0] + acc[1]) + (acc[2] + acc[3]);      // <v, x_t>
        const float sf = (float)sigma;
        const float z = sf * qv;
        if (valid) zrow[(int64_t)t * a.zl.zs_t] = z;
        const float b = (eta * slope<LOSS>(z, y0)) * __builtin_amdgcn_rcpf(sf);
#pragma unroll
        for (int j = 0; j < NZ; ++j)
            if (j < nnz) Vq[off[j]] = fmaf(-b, xv[j], v[j]);

        const double bd = (double)b;
        n2 = fma(bd * bd, (double)X2, fma(-2.0 * bd, (double)qv, n2));
        n2 = n2 > 0.0 ? n2 : 0.0;
        if (sigma * sigma * n2 > D2) sigma = a.D * rsqrt(n2);                        // projection
        if (__any(sigma < kSparseFoldLo)) {
            // fold sigma into the columns of this wavefront and re-measure ||v||^2
            const float s = (float)sigma;
            double m2 = 0.0;
            for (int64_t j = 0; j < a.d; ++j) {
                const float w = Vq[j * a.RKp] * s;
                Vq[j * a.RKp] = w;
                m2 += (double)w * (double)w;
            }
            n2 = m2;
            sigma = 1.0;
        }
        if (lane == 0) *(volatile int *)&progress = t + 1;
        c0 = c1; x0 = x1; y0 = y1;
        c1 = c2; x1 = x2; y1 = y2;
    }
    a.sigma[q] = sigma;
    a.n2[q] = n2;
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

template <int NZ>
hipError_t launch_nz(const SparseArgs &a, int loss, hipStream_t s)
{
    const int nblk = (a.R * a.K + kWave - 1) / kWave;
    switch (loss) {
        case 0: hipLaunchKernelGGL((sparse_rounds_kernel<NZ, 0>), dim3(nblk), dim3(2 * kWave), 0, s, a); break;
        case 1: hipLaunchKernelGGL((sparse_rounds_kernel<NZ, 1>), dim3(nblk), dim3(2 * kWave), 0, s, a); break;
        case 2: hipLaunchKernelGGL((sparse_rounds_kernel<NZ, 2>), dim3(nblk), dim3(2 * kWave), 0, s, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_sparse_rounds(const SparseArgs &a0, int loss, hipStream_t s)
{
    SparseArgs a = a0;
    if (const char *e = getenv("OCO_SPARSE_PREFETCH")) a.prefetch = atoi(e);
    if (a.n <= 0) return hipSuccess;
    const int64_t nthr = (int64_t)a.n * a.R;
    hipLaunchKernelGGL(sparse_comparator_kernel, dim3((unsigned)((nthr + 255) / 256)), dim3(256), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int groups = a.RKp / kWave;
    for (int done = 0; done < a0.n;) {
        const int64_t tabs = a0.t0 + done;
        int len = (int)(kSegment - tabs % kSegment);          // up to the next multiple of kSegment
        if (len > a0.n - done) len = a0.n - done;
        SparseArgs g = a;
        g.col = a.col + (int64_t)done * a.nnz;
        g.val = a.val + (int64_t)done * a.nnz;
        g.y = a.y ? a.y + done : nullptr;
        g.Z = a.Z + (int64_t)done * a.zl.zs_t;
        g.t0 = tabs;
        g.n = len;
        if (a.nnz <= 8) e = launch_nz<8>(g, loss, s);
        else if (a.nnz <= 16) e = launch_nz<16>(g, loss, s);
        else if (a.nnz <= 32) e = launch_nz<32>(g, loss, s);
        else if (a.nnz <= 64) e = launch_nz<64>(g, loss, s);
        else e = hipErrorInvalidValue;
        if (e != hipSuccess) return e;
        done += len;
        if ((a0.t0 + done) % kSegment == 0) {                 // a segment of the horizon ended
            hipLaunchKernelGGL(sparse_fold_kernel, dim3(1024, groups), dim3(256), 0, s, a.V, a.sigma, a.d, a.RKp);
            hipLaunchKernelGGL(sparse_fold_finish_kernel, dim3(groups), dim3(kWave), 0, s, a.sigma, a.n2);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
    }
    return hipSuccess;
}

}  // namespace oco
