// Verification step of speculative decoding (Algorithm 1) on batches of draft / target
// distributions: accepted length, residual resampling, and the acceptance rate of Eq. (1).
//
// Both kernels stream rows of V probabilities from HBM and are bound by that traffic.
// sd_verify reads, per step, 2k gathered scalars and then only the rows it needs: p and q at
// the first rejected position (or p at position k).  One workgroup per step (several resident
// per compute unit, so that one step's gather and search latencies hide behind the others'
// streaming); the row is read once with 16-byte loads, summed per 1024-token
// segment as 64-bit integers (units of 2^-40: integer sums do not
// depend on the order, so the draw is reproducible bit for bit), the segment holding the
// target mass is found from the segment sums, and only that segment is read again to find
// the token.
#include "../../include/specdec.h"

#include <hip/hip_runtime.h>

namespace {

// The verify kernel comes in two workgroup sizes: 256 threads (eight steps resident per compute
// unit) for batches that fill the chip, 1024 threads when there are few steps.
typedef unsigned long long u64;

__device__ __forceinline__ u64 shfl_xor_u64(u64 v, int mask)
{
    const unsigned lo = (unsigned)__shfl_xor((int)(unsigned)v, mask);
    const unsigned hi = (unsigned)__shfl_xor((int)(unsigned)(v >> 32), mask);
    return ((u64)hi << 32) | lo;
}

__device__ __forceinline__ u64 bcast_u64(u64 v, int src)
{
    const unsigned lo = (unsigned)__shfl((int)(unsigned)v, src);
    const unsigned hi = (unsigned)__shfl((int)(unsigned)(v >> 32), src);
    return ((u64)hi << 32) | lo;
}

__device__ __forceinline__ u64 shfl_up_u64(u64 v, int delta)
{
    const unsigned lo = (unsigned)__shfl_up((int)(unsigned)v, delta);
    const unsigned hi = (unsigned)__shfl_up((int)(unsigned)(v >> 32), delta);
    return ((u64)hi << 32) | lo;
}

// the four residual masses of tokens x .. x+3 (x a multiple of 4), in units of 2^-40, as
// integer-valued floats: scaling by 2^40 is exact and v_trunc drops the fraction
__device__ __forceinline__ void load_mass(const float *pr, const float *qr, int x, int V, int vec_ok, float (&f)[4])
{
    float pv[4] = {0.f, 0.f, 0.f, 0.f}, qv[4] = {0.f, 0.f, 0.f, 0.f};
    if (vec_ok) {
        if (x < V) {
            const float4 a = *reinterpret_cast<const float4 *>(pr + x);
            pv[0] = a.x; pv[1] = a.y; pv[2] = a.z; pv[3] = a.w;
            if (qr) {
                const float4 c = *reinterpret_cast<const float4 *>(qr + x);
                qv[0] = c.x; qv[1] = c.y; qv[2] = c.z; qv[3] = c.w;
            }
        }
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (x + e < V) { pv[e] = pr[x + e]; if (qr) qv[e] = qr[x + e]; }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) f[e] = truncf((qr ? fmaxf(0.f, pv[e] - qv[e]) : pv[e]) * 0x1p40f);
}

__device__ __forceinline__ double shfl_xor_f64(double v, int mask)
{
    const u64 b = (u64)__double_as_longlong(v);
    return __longlong_as_double((long long)shfl_xor_u64(b, mask));
}

template <int kThreads>
__global__ void __launch_bounds__(kThreads) sd_verify_kernel(const float *p, const float *q, const int32_t *tok,
                                                             const float *r, const uint32_t *u, int k, int V,
                                                             int vec_ok, int32_t *n_out, int32_t *next_out)
{
    constexpr int kWaves = kThreads / 64;
    constexpr int kSeg = 4 * kThreads;            // tokens per segment: four per thread
    constexpr int kMaxSeg = SD_MAX_V / kSeg;
    __shared__ int n_sh, seg_sh, next_sh;
    constexpr int kUnroll = 4;
    __shared__ u64 seg[kMaxSeg + kUnroll];
    __shared__ u64 wtot[kWaves];
    __shared__ u64 z_sh, base_sh, target_sh;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t b = blockIdx.x;

    // ---- accepted length: the first position whose draft token fails r q <= p -------------
    if (wave == 0) {
        bool rej = false;
        if (lane < k) {
            int t = tok[b * k + lane];
            t = t < 0 ? 0 : (t >= V ? V - 1 : t);
            const float pv = p[(b * (k + 1) + lane) * V + t];
            const float qv = q[(b * k + lane) * V + t];
            rej = !(__fmul_rn(r[b * k + lane], qv) <= pv);
        }
        const u64 mask = __ballot(rej);
        if (lane == 0) { n_sh = mask ? __builtin_ctzll(mask) : k; next_sh = V; }
    }
    __syncthreads();
    const int n = n_sh;
    const float *pr = p + (b * (k + 1) + n) * V;
    const float *qr = n < k ? q + (b * k + n) * V : nullptr;
    const int nseg = (V + kSeg - 1) / kSeg;

    for (int attempt = 0; attempt < 2; ++attempt) {
        for (int s = tid; s < nseg; s += kThreads) seg[s] = 0;
        __syncthreads();
        // ---- one pass over the row: integer mass of every segment of kSeg tokens ------------
        // (a wavefront's share of a segment is < 2^49 units, so float64 sums of the integer
        // masses are exact and their order is immaterial)
        for (int s0 = 0; s0 < nseg; s0 += kUnroll) {       // kUnroll segments (2 kUnroll loads) in flight
            float f[kUnroll][4];
#pragma unroll
            for (int w = 0; w < kUnroll; ++w)                   // past the row: zeros
                load_mass(pr, qr, (s0 + w) * kSeg + tid * 4, V, vec_ok, f[w]);
            double t[kUnroll];
#pragma unroll
            for (int w = 0; w < kUnroll; ++w)
                t[w] = ((double)f[w][0] + (double)f[w][1]) + ((double)f[w][2] + (double)f[w][3]);
#pragma unroll
            for (int sh = 32; sh >= 1; sh >>= 1)
#pragma unroll
                for (int w = 0; w < kUnroll; ++w) t[w] += shfl_xor_f64(t[w], sh);
            if (lane == 0)
#pragma unroll
                for (int w = 0; w < kUnroll; ++w)
                    if (t[w] != 0.0) atomicAdd(&seg[s0 + w], (u64)t[w]);   // s0 + w < nseg + kUnroll: seg has the room
        }
        __syncthreads();
        // ---- total mass, target, and the segment that holds it (wavefront 0) ---------------
        if (wave == 0) {
            u64 loc[kMaxSeg / 64];
            u64 run = 0;
#pragma unroll
            for (int c = 0; c < kMaxSeg / 64; ++c) {
                const int s = lane * (kMaxSeg / 64) + c;
                run += s < nseg ? seg[s] : 0;
                loc[c] = run;                      // inclusive within the lane's block
            }
            u64 incl = run;                        // inclusive scan of the lane totals
#pragma unroll
            for (int sh = 1; sh < 64; sh <<= 1) {
                const u64 o = shfl_up_u64(incl, sh);
                if (lane >= sh) incl += o;
            }
            const u64 Z = bcast_u64(incl, 63);
            const u64 target = __umul64hi(Z, (u64)u[b] << 32);       // floor(Z u / 2^32) < Z
            const u64 excl = incl - run;
            // the first segment whose inclusive prefix exceeds the target
            int found = -1;
            u64 base = 0;
#pragma unroll
            for (int c = kMaxSeg / 64 - 1; c >= 0; --c) {
                const u64 before = excl + (c ? loc[c - 1] : 0);
                if (excl + loc[c] > target && before <= target) { found = lane * (kMaxSeg / 64) + c; base = before; }
            }
            if (found >= 0) { seg_sh = found; base_sh = base; }       // exactly one lane if Z > 0
            if (lane == 0) { z_sh = Z; target_sh = target; }
        }
        __syncthreads();
        if (z_sh != 0 || !qr) break;
        qr = nullptr;                               // the residual vanished at this resolution: p' = p_n
        __syncthreads();
    }
    if (z_sh == 0) {                                // an all-zero target row: nothing to draw
        if (tid == 0) { n_out[b] = n; next_out[b] = 0; }
        return;
    }
    // ---- second look at one segment: the token at which the prefix passes the target --------
    {
        const int x = seg_sh * kSeg + tid * 4;
        float ff[4];
        load_mass(pr, qr, x, V, vec_ok, ff);
        u64 f[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) f[e] = (u64)ff[e];
        const u64 mine = (f[0] + f[1]) + (f[2] + f[3]);
        u64 incl = mine;
#pragma unroll
        for (int sh = 1; sh < 64; sh <<= 1) {
            const u64 o = shfl_up_u64(incl, sh);
            if (lane >= sh) incl += o;
        }
        if (lane == 63) wtot[wave] = incl;
        __syncthreads();
        u64 before = base_sh + incl - mine;
        for (int w = 0; w < wave; ++w) before += wtot[w];
        const u64 target = target_sh;
        if (before <= target && before + mine > target) {          // exactly one thread
            int e = 0;
            u64 c = before + f[0];
            while (c <= target) { ++e; c += f[e]; }
            next_sh = x + e;
        }
        __syncthreads();
        if (tid == 0) { n_out[b] = n; next_out[b] = next_sh; }
    }
}

// acc[b][j] = sum_x min(p_j(x), q_j(x)); one workgroup per row pair, float64 sums, fixed order
__global__ void __launch_bounds__(256) sd_acceptance_kernel(const float *p, const float *q, int k, int V,
                                                            int vec_ok, double *acc)
{
    __shared__ double part[4];
    const int64_t b = blockIdx.x / k;
    const int j = blockIdx.x % k;
    const float *pr = p + (b * (k + 1) + j) * V;
    const float *qr = q + (b * k + j) * V;
    double a0 = 0.0, a1 = 0.0;
    if (vec_ok) {
        const float4 *p4 = reinterpret_cast<const float4 *>(pr);
        const float4 *q4 = reinterpret_cast<const float4 *>(qr);
        const int n4 = V / 4;
        int e = threadIdx.x;
        for (; e + 768 < n4; e += 1024) {          // four independent 16-byte loads per stream in flight
            float4 a[4], c[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) { a[w] = p4[e + 256 * w]; c[w] = q4[e + 256 * w]; }
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                a0 += (double)fminf(a[w].x, c[w].x) + (double)fminf(a[w].y, c[w].y);
                a1 += (double)fminf(a[w].z, c[w].z) + (double)fminf(a[w].w, c[w].w);
            }
        }
        for (; e < n4; e += 256) {
            const float4 a = p4[e], c = q4[e];
            a0 += (double)fminf(a.x, c.x) + (double)fminf(a.y, c.y);
            a1 += (double)fminf(a.z, c.z) + (double)fminf(a.w, c.w);
        }
    } else {
        for (int e = threadIdx.x; e < V; e += 256) a0 += (double)fminf(pr[e], qr[e]);
    }
    double s = a0 + a1;
#pragma unroll
    for (int sh = 32; sh >= 1; sh >>= 1) {
        const unsigned lo = (unsigned)__shfl_xor((int)(unsigned)__double_as_longlong(s), sh);
        const unsigned hi = (unsigned)__shfl_xor((int)(unsigned)((u64)__double_as_longlong(s) >> 32), sh);
        s += __longlong_as_double((long long)(((u64)hi << 32) | lo));
    }
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
    __syncthreads();
    if (threadIdx.x == 0) acc[b * k + j] = (part[0] + part[1]) + (part[2] + part[3]);
}

bool misaligned(const void *p, unsigned a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

int check_sizes(int64_t B, int64_t k, int64_t V)
{
    if (B <= 0 || k <= 0 || V <= 0) return SD_EINVAL;
    if (k > SD_MAX_K || V > SD_MAX_V || B > (1 << 30)) return SD_EUNSUPPORTED;
    return SD_OK;
}

}  // namespace

extern "C" {

int sd_verify(const float *p_dev, const float *q_dev, const int32_t *tok_dev, const float *r_dev,
              const uint32_t *u_dev, int64_t B, int64_t k, int64_t V, int32_t *n_dev, int32_t *next_dev,
              void *hip_stream)
{
    if (!p_dev || !q_dev || !tok_dev || !r_dev || !u_dev || !n_dev || !next_dev) return SD_EINVAL;
    if (misaligned(p_dev, 4) || misaligned(q_dev, 4) || misaligned(tok_dev, 4) || misaligned(r_dev, 4) ||
        misaligned(u_dev, 4) || misaligned(n_dev, 4) || misaligned(next_dev, 4))
        return SD_EINVAL;
    const int rc = check_sizes(B, k, V);
    if (rc != SD_OK) return rc;
    const int vec_ok = (V % 4 == 0) && !misaligned(p_dev, 16) && !misaligned(q_dev, 16);
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    if (B >= 1024)
        hipLaunchKernelGGL(sd_verify_kernel<256>, dim3((unsigned)B), dim3(256), 0, s, p_dev, q_dev, tok_dev, r_dev,
                           u_dev, (int)k, (int)V, vec_ok, n_dev, next_dev);
    else
        hipLaunchKernelGGL(sd_verify_kernel<1024>, dim3((unsigned)B), dim3(1024), 0, s, p_dev, q_dev, tok_dev, r_dev,
                           u_dev, (int)k, (int)V, vec_ok, n_dev, next_dev);
    return hipGetLastError() == hipSuccess ? SD_OK : SD_EHIP;
}

int sd_acceptance(const float *p_dev, const float *q_dev, int64_t B, int64_t k, int64_t V, double *acc_dev,
                  void *hip_stream)
{
    if (!p_dev || !q_dev || !acc_dev) return SD_EINVAL;
    if (misaligned(p_dev, 4) || misaligned(q_dev, 4) || misaligned(acc_dev, 8)) return SD_EINVAL;
    const int rc = check_sizes(B, k, V);
    if (rc != SD_OK) return rc;
    if (B * k > 0x7fffffffLL) return SD_EUNSUPPORTED;
    const int vec_ok = (V % 4 == 0) && !misaligned(p_dev, 16) && !misaligned(q_dev, 16);
    hipLaunchKernelGGL(sd_acceptance_kernel, dim3((unsigned)(B * k)), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), p_dev, q_dev, (int)k, (int)V, vec_ok, acc_dev);
    return hipGetLastError() == hipSuccess ? SD_OK : SD_EHIP;
}

const char *sd_strerror(int status)
{
    switch (status) {
        case SD_OK: return "ok";
        case SD_EINVAL: return "invalid argument";
        case SD_EUNSUPPORTED: return "size not supported by the kernels";
        case SD_EHIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

}  // extern "C"
