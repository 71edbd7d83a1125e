// Meta learner and regret (Sec. 3.3 Hedge weights, Eq. (2) regret), state
// export and state initialisation.
//
// The round kernels leave z_t^i = <w_t^i, x_t> (i < K) and z_t^u = <u_t, x_t>
// in Z for the n rounds of a call.  Everything here is float64 on a handful of
// scalars per round:
//     l_t^i = phi(z_t^i; y_t)                       base losses
//     L_t^i = L_{t-1}^i + l_{t-1}^i                 (running sum, strictly in round order)
//     p_t^i = exp(-eps L_t^i) / sum_j exp(-eps L_t^j)
//     <w_t, x_t> = sum_i p_t^i z_t^i                (w_t = sum_i p_t^i w_t^i is linear in w)
//     regret += phi(<w_t, x_t>; y_t) - phi(z_t^u; y_t)
// With the meta learner's hint (optimism at both levels of the ensemble: Hedge on the cumulative
// losses plus a guess of the coming loss, the last observed one) the exponent of round t is
// L_t^i + l_{t-1}^i instead; the last loss of a call is kept in the state for the next call.
// One workgroup per run walks the rounds in tiles: losses of a tile in
// parallel over rounds, the running sums by K threads in round order, the
// weights and the regret terms in parallel over rounds, and the regret sum by
// one thread in round order -- so the result does not depend on how the
// horizon is cut into calls.
#include "oco_internal.h"

namespace oco {
namespace {

template <int LOSS> __device__ __forceinline__ double phi(double z, double y)
{
    if (LOSS == 0) return z;
    if (LOSS == 1) { const double e = z - y; return e * e; }
    // log(1 + exp(-m)) without overflow: log1p(exp(-|m|)) + max(-m, 0).  One exp and one log1p
    // for every lane (a branch on the sign of m would run both sides in most wavefronts).
    const double m = y * z;
    const double am = fabs(m);
    const double lp = log1p(exp(-am));
    return m > 0.0 ? lp : lp + am;
}

template <int LOSS>
__global__ void __launch_bounds__(256) meta_kernel(const MetaArgs a)
{
    extern __shared__ double sm[];
    const int TM = blockDim.x;
    const int K = a.K;
    double *lmat = sm;                 // [TM][K]: losses, then cumulative losses before the round
    double *diff = sm + (size_t)TM * K; // [TM]
    const int r = blockIdx.x;
    const int j = threadIdx.x;
    const float *Zr = a.Z + (int64_t)r * a.zl.zs_r;
    const float *yrow = a.y ? a.y + (int64_t)r * a.y_run_stride : nullptr;

    double Lacc = (j < K) ? a.L[(int64_t)r * K + j] : 0.0;   // thread i < K carries L^i
    const bool hint = a.last != nullptr;
    double lprev = (hint && j < K) ? a.last[(int64_t)r * K + j] : 0.0;   // ... and the last loss l_{t-1}^i
    double reg = (j == 0) ? a.regret[r] : 0.0;

    for (int t0 = 0; t0 < a.n; t0 += TM) {
        const int cnt = min(TM, a.n - t0);
        const int t = t0 + j;
        double yt = 0.0;
        if (j < cnt) {
            yt = yrow ? (double)yrow[t] : 0.0;
            for (int i = 0; i < K; ++i) {
                const double z = (double)Zr[(int64_t)i * a.zl.zs_i + (int64_t)t * a.zl.zs_t];
                lmat[j * K + i] = phi<LOSS>(z, yt);
            }
        }
        __syncthreads();
        if (j < K) {
            // running sums in round order; whole chunks issue their LDS reads together (one
            // dependent LDS round trip per chunk instead of per round), the tail goes one by one
            int jj = 0;
            for (; jj + 16 <= cnt; jj += 16) {
                double v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = lmat[(jj + u) * K + j];
#pragma unroll
                for (int u = 0; u < 16; ++u) {
                    const double l = v[u];
                    v[u] = hint ? Lacc + lprev : Lacc;
                    Lacc += l;
                    lprev = l;
                }
#pragma unroll
                for (int u = 0; u < 16; ++u) lmat[(jj + u) * K + j] = v[u];
            }
            for (; jj < cnt; ++jj) {
                const double l = lmat[jj * K + j];
                lmat[jj * K + j] = hint ? Lacc + lprev : Lacc;
                Lacc += l;
                lprev = l;
            }
        }
        __syncthreads();
        if (j < cnt) {
            double Lmin = lmat[j * K];
            for (int i = 1; i < K; ++i) Lmin = fmin(Lmin, lmat[j * K + i]);
            double S = 0.0, zs = 0.0;
            for (int i = 0; i < K; ++i) {
                const double e = exp(-a.eps * (lmat[j * K + i] - Lmin));
                const double z = (double)Zr[(int64_t)i * a.zl.zs_i + (int64_t)t * a.zl.zs_t];
                S += e;
                zs += e * z;
            }
            const double zhat = zs / S;
            const double zu = (double)Zr[(int64_t)K * a.zl.zs_i + (int64_t)t * a.zl.zs_t];
            diff[j] = phi<LOSS>(zhat, yt) - phi<LOSS>(zu, yt);
        }
        __syncthreads();
        if (j == 0)
        {
            int jj = 0;
            for (; jj + 16 <= cnt; jj += 16) {
                double v[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) v[u] = diff[jj + u];
#pragma unroll
                for (int u = 0; u < 16; ++u) reg += v[u];
            }
            for (; jj < cnt; ++jj) reg += diff[jj];
        }
        // lmat/diff are rewritten only after the next tile's first barrier
    }
    if (j < K) a.L[(int64_t)r * K + j] = Lacc;
    if (hint && j < K) a.last[(int64_t)r * K + j] = lprev;
    if (j == 0) a.regret[r] = reg;
}

// p = softmax(-eps L) of one run, into shared memory (first K threads)
// (last: the meta learner's hint, the last observed losses, or null)
__device__ void hedge_weights(const double *L, const double *last, int K, double eps, double *p_sh)
{
    if (threadIdx.x == 0) {
        double Lmin = L[0] + (last ? last[0] : 0.0);
        for (int i = 1; i < K; ++i) Lmin = fmin(Lmin, L[i] + (last ? last[i] : 0.0));
        double S = 0.0;
        for (int i = 0; i < K; ++i) { p_sh[i] = exp(-eps * (L[i] + (last ? last[i] : 0.0) - Lmin)); S += p_sh[i]; }
        for (int i = 0; i < K; ++i) p_sh[i] /= S;
    }
    __syncthreads();
}

// dense layout: V[R][K][d], sigma float [R][K].  Optimistic mode: V holds the intermediate
// model and the iterate handed out is the one played next, Proj[sigma V - ha x_last] (Eq. (3)).
__global__ void __launch_bounds__(256) export_dense_kernel(const ExportArgs a)
{
    __shared__ double p_sh[64];
    __shared__ float s_sh[64], h_sh[64], f_sh[64];
    const int r = blockIdx.y;
    const int K = a.K;
    hedge_weights(a.L + (int64_t)r * K, a.last ? a.last + (int64_t)r * K : nullptr, K, a.eps, p_sh);
    if (threadIdx.x < K) {
        const int64_t q = (int64_t)r * K + threadIdx.x;
        const float sg = static_cast<const float *>(a.sigma)[q];
        float ha = 0.f, f = 1.f;
        if (a.optimistic) {
            ha = a.ha[q];
            const double x2l = (double)a.x2last[a.x_shared ? 0 : r];
            const double m = fma((double)ha * (double)ha, x2l,
                                 fma(-2.0 * (double)ha, (double)a.hp[q], (double)sg * (double)sg * a.n2[q]));
            const float mf = (float)m;
            if (mf > a.D * a.D) f = a.D * __builtin_amdgcn_rsqf(mf);
        }
        s_sh[threadIdx.x] = sg; h_sh[threadIdx.x] = ha; f_sh[threadIdx.x] = f;
    }
    __syncthreads();
    if (a.p && blockIdx.x == 0 && threadIdx.x < K) a.p[(int64_t)r * K + threadIdx.x] = (float)p_sh[threadIdx.x];
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= a.d) return;
    const float xl = a.optimistic ? a.xlast[(a.x_shared ? 0 : (int64_t)r * a.d) + j] : 0.f;
    double acc = 0.0;
    for (int i = 0; i < K; ++i) {
        float w = s_sh[i] * a.V[((int64_t)r * K + i) * a.d + j];
        if (a.optimistic) w = f_sh[i] * fmaf(-h_sh[i], xl, w);
        if (a.W) a.W[((int64_t)r * K + i) * a.d + j] = w;
        acc += p_sh[i] * (double)w;
    }
    if (a.wbar) a.wbar[(int64_t)r * a.d + j] = (float)acc;
}

// sparse layout: V[d][RKp], sigma double [RKp].  64x64 transpose through LDS:
// rows = coordinates, columns = learners.
// optimistic mode: scale f and hint coefficient ha of the iterate played next, Proj[sigma v - ha x_last]
__device__ __forceinline__ void played_scale(const ExportArgs &a, int q, double sg, float &f, float &ha)
{
    f = 1.f;
    ha = 0.f;
    if (!a.optimistic) return;
    ha = a.ha[q];
    const double m = fma((double)ha * (double)ha, (double)a.x2last[q],
                         fma(-2.0 * (double)ha, (double)a.hp[q], sg * sg * a.n2[q]));
    const float mf = (float)m;
    if (mf > a.D * a.D) f = a.D * __builtin_amdgcn_rsqf(mf);
}

__global__ void __launch_bounds__(256) export_sparse_W_kernel(const ExportArgs a)
{
    __shared__ float tile[64][65];
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    const int64_t j0 = (int64_t)blockIdx.x * 64;
    const int q0 = blockIdx.y * 64;
    const int nq = a.R * a.K;
    const double *sg = static_cast<const double *>(a.sigma);
    const float s = (q0 + tx < nq) ? (float)sg[q0 + tx] : 0.f;
    float f = 1.f, ha = 0.f;
    if (q0 + tx < nq) played_scale(a, q0 + tx, sg[q0 + tx], f, ha);
    for (int row = ty; row < 64; row += 4) {
        const int64_t j = j0 + row;
        float v = 0.f;
        if (j < a.d && q0 + tx < nq) {
            v = (float)((double)a.V[j * a.RKp + q0 + tx] * (double)s);
            if (a.optimistic) v = f * fmaf(-ha, a.xlast[j], v);
        }
        tile[row][tx] = v;
    }
    __syncthreads();
    for (int tq = ty; tq < 64; tq += 4) {
        const int q = q0 + tq;
        const int64_t j = j0 + tx;
        if (q < nq && j < a.d) a.W[(int64_t)q * a.d + j] = tile[tx][tq];
    }
}

// p and wbar for a chunk of 16 runs and a tile of 64 coordinates per workgroup.  Threads walk
// the tile with the run index fastest, so a wavefront reads whole row segments of V (the K
// learners of 16 runs lie next to each other); the sums go through LDS and are written with
// the coordinate fastest.  Sum over learners in the order i = 0..K-1, float64.
constexpr int kExpRuns = 16, kExpRows = 64;
__global__ void __launch_bounds__(256) export_sparse_p_wbar_kernel(const ExportArgs a)
{
    __shared__ double p_sh[kExpRuns][64];
    __shared__ float s_sh[kExpRuns][64], f_sh[kExpRuns][64], h_sh[kExpRuns][64];
    __shared__ float tile[kExpRows][kExpRuns + 1];
    const int K = a.K;
    const int r0 = blockIdx.y * kExpRuns;
    const int64_t j0 = (int64_t)blockIdx.x * kExpRows;
    if (threadIdx.x < kExpRuns && r0 + (int)threadIdx.x < a.R) {
        const int rl = threadIdx.x, r = r0 + rl;
        const double *L = a.L + (int64_t)r * K;
        const double *last = a.last ? a.last + (int64_t)r * K : nullptr;      // the meta learner's hint
        double Lmin = L[0] + (last ? last[0] : 0.0);
        for (int i = 1; i < K; ++i) Lmin = fmin(Lmin, L[i] + (last ? last[i] : 0.0));
        double S = 0.0;
        for (int i = 0; i < K; ++i) { p_sh[rl][i] = exp(-a.eps * (L[i] + (last ? last[i] : 0.0) - Lmin)); S += p_sh[rl][i]; }
        for (int i = 0; i < K; ++i) {
            p_sh[rl][i] /= S;
            const double sg = static_cast<const double *>(a.sigma)[r * K + i];
            s_sh[rl][i] = (float)sg;
            played_scale(a, r * K + i, sg, f_sh[rl][i], h_sh[rl][i]);
            if (a.p && blockIdx.x == 0) a.p[(int64_t)r * K + i] = (float)p_sh[rl][i];
        }
    }
    __syncthreads();
    if (!a.wbar) return;
    for (int idx = threadIdx.x; idx < kExpRows * kExpRuns; idx += 256) {
        const int rl = idx % kExpRuns, row = idx / kExpRuns;
        const int r = r0 + rl;
        const int64_t j = j0 + row;
        double acc = 0.0;
        if (r < a.R && j < a.d) {
            const float xl = a.optimistic ? a.xlast[j] : 0.f;
            const float *v = a.V + j * a.RKp + (int64_t)r * K;
            for (int i = 0; i < K; ++i) {
                float w = (float)((double)v[i] * (double)s_sh[rl][i]);
                if (a.optimistic) w = f_sh[rl][i] * fmaf(-h_sh[rl][i], xl, w);
                acc += p_sh[rl][i] * (double)w;
            }
        }
        tile[row][rl] = (float)acc;
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < kExpRows * kExpRuns; idx += 256) {
        const int row = idx % kExpRows, rl = idx / kExpRows;
        const int r = r0 + rl;
        const int64_t j = j0 + row;
        if (r < a.R && j < a.d) a.wbar[(int64_t)r * a.d + j] = tile[row][rl];
    }
}

__global__ void __launch_bounds__(256) zero_kernel(uint4 *p, size_t n16)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < n16; k += stride)
        p[k] = make_uint4(0u, 0u, 0u, 0u);
}

__global__ void __launch_bounds__(256) ones_kernel(void *p, int64_t n, int is_double)
{
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k >= n) return;
    if (is_double) static_cast<double *>(p)[k] = 1.0; else static_cast<float *>(p)[k] = 1.0f;
}

// Lemma 1 / Theorem 1, one thread per run
__global__ void __launch_bounds__(256) accel_bounds_kernel(const double *regret, int R, double t, double k,
                                                           double alpha, double *out)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= R) return;
    const double reg = regret[r] > 0.0 ? regret[r] : 0.0;
    const double k1 = k + 1.0;
    const double lo = k1 * t / (1.0 + k1 * sqrt(reg / (2.0 * t)));
    out[4 * r + 0] = lo;
    out[4 * r + 1] = k1 * t;
    out[4 * r + 2] = lo / (t * (alpha * k + 1.0));
    out[4 * r + 3] = k1 / (alpha * k + 1.0);
}

}  // namespace

hipError_t launch_meta(const MetaArgs &a, int loss, hipStream_t s)
{
    if (a.n <= 0) return hipSuccess;
    const int TM = a.K <= 24 ? 256 : 64;
    const size_t smem = sizeof(double) * ((size_t)TM * a.K + TM);
    switch (loss) {
        case 0: hipLaunchKernelGGL(meta_kernel<0>, dim3(a.R), dim3(TM), smem, s, a); break;
        case 1: hipLaunchKernelGGL(meta_kernel<1>, dim3(a.R), dim3(TM), smem, s, a); break;
        case 2: hipLaunchKernelGGL(meta_kernel<2>, dim3(a.R), dim3(TM), smem, s, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_export(const ExportArgs &a, hipStream_t s)
{
    if (!a.W && !a.p && !a.wbar) return hipSuccess;
    if (!a.sparse) {
        dim3 grid((a.d + 255) / 256, a.R);
        hipLaunchKernelGGL(export_dense_kernel, grid, dim3(256), 0, s, a);
        return hipGetLastError();
    }
    if (a.W) {
        dim3 grid((unsigned)(((int64_t)a.d + 63) / 64), (a.R * a.K + 63) / 64);
        hipLaunchKernelGGL(export_sparse_W_kernel, grid, dim3(256), 0, s, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (a.p || a.wbar) {
        dim3 grid(a.wbar ? (unsigned)(((int64_t)a.d + kExpRows - 1) / kExpRows) : 1u,
                  (unsigned)((a.R + kExpRuns - 1) / kExpRuns));
        hipLaunchKernelGGL(export_sparse_p_wbar_kernel, grid, dim3(256), 0, s, a);
        return hipGetLastError();
    }
    return hipSuccess;
}

hipError_t launch_accel_bounds(const double *regret, int R, int64_t t, int64_t k, double alpha, double *out,
                               hipStream_t s)
{
    hipLaunchKernelGGL(accel_bounds_kernel, dim3((R + 255) / 256), dim3(256), 0, s, regret, R, (double)t,
                       (double)k, alpha, out);
    return hipGetLastError();
}

__global__ void __launch_bounds__(64) set_eta_kernel(float *eta, const EtaTable tab, int K)
{
    if ((int)threadIdx.x < K) eta[threadIdx.x] = tab.v[threadIdx.x];
}

hipError_t launch_set_eta(float *eta_dev, const EtaTable &tab, int K, hipStream_t s)
{
    hipLaunchKernelGGL(set_eta_kernel, dim3(1), dim3(64), 0, s, eta_dev, tab, K);
    return hipGetLastError();
}

hipError_t launch_init_state(void *zero_base, size_t zero_bytes, void *sigma, int64_t n_sigma,
                             int sigma_is_double, hipStream_t s)
{
    const size_t n16 = zero_bytes / 16;
    if (n16) {
        const unsigned blocks = (unsigned)((n16 + 255) / 256 < 4096 ? (n16 + 255) / 256 : 4096);
        hipLaunchKernelGGL(zero_kernel, dim3(blocks), dim3(256), 0, s, static_cast<uint4 *>(zero_base), n16);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (n_sigma) {
        hipLaunchKernelGGL(ones_kernel, dim3((unsigned)((n_sigma + 255) / 256)), dim3(256), 0, s, sigma,
                           n_sigma, sigma_is_double);
        return hipGetLastError();
    }
    return hipSuccess;
}

}  // namespace oco
