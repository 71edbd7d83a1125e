// Sparse rounds of the base learners (Sec. 3.1 update inside the ensemble of
// Sec. 3.3) for a high-dimensional iterate that lives in HBM.
//
// A round with nnz non-zero features touches nnz coordinates of every
// learner: the gradient step changes only those, and the projection onto the
// ball is a rescaling, carried by a per-learner scalar (w = sigma * v), so a
// round never sweeps the d coordinates.  ||v||^2 is carried in float64 and
// advanced by the exact change of the touched coordinates,
// sum_j (v'_j^2 - v_j^2), which keeps it equal to the norm of the stored
// float32 vector up to float64 rounding.
//
// Layout.  The round stream is shared by all runs, so every learner of every
// run touches the SAME coordinates in a round.  V is stored coordinate-major
// with the R*K learners interleaved, V[j][q], q = r*K + i: the 64 lanes of a
// wavefront are 64 learners, one coordinate of all of them is one contiguous
// 256-byte row segment, every gather and scatter is fully coalesced and all
// the per-learner scalar work (slope, step, norm, projection) runs
// lane-parallel with no reduction.
//
// sigma is folded into v (one sweep over the wavefront's columns) when any
// lane's sigma drops below 2^-40; the sweep also recomputes ||v||^2 exactly.
#include "oco_internal.h"

namespace oco {
namespace {

template <int LOSS> __device__ __forceinline__ float slope(float z, float y)
{
    if (LOSS == 0) return 1.0f;
    if (LOSS == 1) return 2.0f * (z - y);
    return -y / (1.0f + expf(y * z));
}

constexpr double kSparseFoldLo = 0x1p-40;

// NZ: compile-time bound on the entries per round (nnz <= NZ)
template <int NZ, int LOSS>
__global__ void __launch_bounds__(kWave) sparse_rounds_kernel(const SparseArgs a)
{
    const int lane = threadIdx.x;
    const int nq = a.R * a.K;
    const int nblk_learn = (nq + kWave - 1) / kWave;
    const int nnz = a.nnz;
    const int n = a.n;

    if ((int)blockIdx.x >= nblk_learn) {
        // ---- comparator wavefronts: lane = run, z_u[t] = <u_t, x_t> -------------
        const int r = ((int)blockIdx.x - nblk_learn) * kWave + lane;
        if (r >= a.R) return;
        int seg = 0;
        while (seg + 1 < a.S && a.seg_start[seg + 1] <= a.t0) ++seg;
        int64_t next_seg = seg + 1 < a.S ? a.seg_start[seg + 1] : INT64_MAX;
        const float *uu = a.u + ((int64_t)r * a.S + seg) * a.d;
        for (int t = 0; t < n; ++t) {
            if (a.t0 + t == next_seg) {
                ++seg;
                next_seg = seg + 1 < a.S ? a.seg_start[seg + 1] : INT64_MAX;
                uu = a.u + ((int64_t)r * a.S + seg) * a.d;
            }
            const int32_t *ct = a.col + (int64_t)t * nnz;
            const float *vt = a.val + (int64_t)t * nnz;
            float acc = 0.f;
            for (int j = 0; j < nnz; ++j) acc = fmaf(uu[ct[j]], vt[j], acc);
            a.Z[(int64_t)r * a.zl.zs_r + (int64_t)a.K * a.zl.zs_i + (int64_t)t * a.zl.zs_t] = acc;
        }
        return;
    }

    // ---- learner wavefronts: lane = learner q = r*K + i ---------------------------
    const int q = blockIdx.x * kWave + lane;
    const bool valid = q < nq;
    const int qq = valid ? q : 0;
    const int r = qq / a.K, i = qq % a.K;
    const float eta = a.eta[i];
    double sigma = a.sigma[blockIdx.x * kWave + lane];
    double n2 = a.n2[blockIdx.x * kWave + lane];
    const double D2 = a.D * a.D;
    float *Vq = a.V + blockIdx.x * kWave + lane;      // column of this lane (padded columns exist)
    const float *yrow = a.y ? a.y + (int64_t)r * a.y_run_stride : nullptr;
    float *zrow = a.Z + (int64_t)r * a.zl.zs_r + (int64_t)i * a.zl.zs_i;

    for (int t = 0; t < n; ++t) {
        const int32_t *ct = a.col + (int64_t)t * nnz;
        const float *vt = a.val + (int64_t)t * nnz;
        float v[NZ], xv[NZ];
        int64_t off[NZ];
#pragma unroll
        for (int j = 0; j < NZ; ++j) {
            if (j < nnz) {
                off[j] = (int64_t)ct[j] * a.RKp;
                xv[j] = vt[j];
                v[j] = Vq[off[j]];
            } else { off[j] = 0; xv[j] = 0.f; v[j] = 0.f; }
        }
        float acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < NZ; ++j) acc[j & 3] = fmaf(v[j], xv[j], acc[j & 3]);
        const float q0 = (acc[0] + acc[1]) + (acc[2] + acc[3]);
        const float z = (float)(sigma * (double)q0);
        if (valid) zrow[(int64_t)t * a.zl.zs_t] = z;
        const float yt = yrow ? yrow[t] : 0.f;
        const float c = slope<LOSS>(z, yt);
        const float b = (float)((double)(eta * c) / sigma);
        double dn = 0.0;
#pragma unroll
        for (int j = 0; j < NZ; ++j) {
            if (j < nnz) {
                const float vn = fmaf(-b, xv[j], v[j]);
                dn += (double)vn * (double)vn - (double)v[j] * (double)v[j];
                Vq[off[j]] = vn;
            }
        }
        n2 += dn;
        if (sigma * sigma * n2 > D2) sigma = a.D / sqrt(n2);      // projection onto the ball
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
    }
    a.sigma[blockIdx.x * kWave + lane] = sigma;
    a.n2[blockIdx.x * kWave + lane] = n2;
}

template <int NZ>
hipError_t launch_nz(const SparseArgs &a, int loss, hipStream_t s)
{
    const int nblk = (a.R * a.K + kWave - 1) / kWave + (a.R + kWave - 1) / kWave;
    switch (loss) {
        case 0: hipLaunchKernelGGL((sparse_rounds_kernel<NZ, 0>), dim3(nblk), dim3(kWave), 0, s, a); break;
        case 1: hipLaunchKernelGGL((sparse_rounds_kernel<NZ, 1>), dim3(nblk), dim3(kWave), 0, s, a); break;
        case 2: hipLaunchKernelGGL((sparse_rounds_kernel<NZ, 2>), dim3(nblk), dim3(kWave), 0, s, a); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_sparse_rounds(const SparseArgs &a, int loss, hipStream_t s)
{
    if (a.n <= 0) return hipSuccess;
    if (a.nnz <= 8) return launch_nz<8>(a, loss, s);
    if (a.nnz <= 16) return launch_nz<16>(a, loss, s);
    if (a.nnz <= 32) return launch_nz<32>(a, loss, s);
    if (a.nnz <= 64) return launch_nz<64>(a, loss, s);
    return hipErrorInvalidValue;
}

}  // namespace oco
