// Comparator predictions of Eq. (2) for a shared dense round stream.
//
// With one round stream for all runs, the predictions of the comparators,
//     z_t^u[r] = <u_t[r], x_t>,     u_t[r] = the comparator of run r in the segment that holds t,
// are a dense contraction: within one comparator segment, Z^u = U X^T with U the R x d matrix
// of the runs' comparators and X the n x d block of round rows.  It runs on the matrix cores
// (fp32 MFMA 32x32x2, products and sums in float32), apart from the round kernel, whose
// wavefronts then all carry base learners.
//
// Tiling.  A workgroup of four wavefronts computes 64 runs x 64 rounds; wavefront w owns the
// 32 x 32 block (w / 2, w % 2).  The depth d is taken in chunks of kKC coordinates staged in
// LDS (rows padded against bank conflicts, coordinates past d and rows past R or n as zeros).
// One MFMA consumes two depth indices, one per half of the wavefront; so that every lane
// reads 16 contiguous bytes, half h of the wavefront takes the depth indices
// 8 j + 4 h .. 8 j + 4 h + 3 of a chunk in four consecutive MFMAs -- the order of the terms of
// an inner product is free, and it is the same for every output whatever the call boundaries
// are, so results do not depend on how the horizon is cut.
//
// A tile of rounds that straddles a segment boundary is computed once per segment it touches;
// each pass writes only the rounds of its own segment.
#include "oco_internal.h"

namespace oco {
namespace {

constexpr int kTileRuns = 64, kTileRounds = 64;
constexpr int kKC = 64;            // depth coordinates per LDS chunk
constexpr int kRow = kKC + 4;      // padded row length in floats (keeps 16-byte alignment)

typedef float floatx16 __attribute__((ext_vector_type(16)));

template <bool VEC>
__global__ void __launch_bounds__(256) comparator_gemm_kernel(ComparatorGemmArgs a)
{
    __shared__ __attribute__((aligned(16))) float us[kTileRuns * kRow];
    __shared__ __attribute__((aligned(16))) float xs[kTileRounds * kRow];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int tb = blockIdx.x * kTileRounds;           // first round of the tile (relative)
    const int rb = blockIdx.y * kTileRuns;             // first run of the tile
    const int d = a.d;

    // segments touched by the rounds of this tile
    const int64_t t_first = a.t0 + tb;
    const int64_t t_last = a.t0 + min(tb + kTileRounds, a.n) - 1;
    int s_lo = 0;
    while (s_lo + 1 < a.S && a.seg_start[s_lo + 1] <= t_first) ++s_lo;
    int s_hi = s_lo;
    while (s_hi + 1 < a.S && a.seg_start[s_hi + 1] <= t_last) ++s_hi;

    const int half = lane >> 5;                        // which of the two depth indices of an MFMA
    const int l32 = lane & 31;
    const float *ua = us + ((wave >> 1) * 32 + l32) * kRow + 4 * half;
    const float *xa = xs + ((wave & 1) * 32 + l32) * kRow + 4 * half;

    for (int s = s_lo; s <= s_hi; ++s) {
        floatx16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;

        for (int kc = 0; kc < d; kc += kKC) {
            // stage 64 rows x kKC coordinates of U (segment s) and of X
            if (VEC) {
#pragma unroll
                for (int e = tid; e < kTileRuns * (kKC / 4); e += 256) {
                    const int row = e / (kKC / 4), j = (e % (kKC / 4)) * 4;
                    float4 uv = make_float4(0.f, 0.f, 0.f, 0.f), xv = uv;
                    if (kc + j < d) {
                        if (rb + row < a.R)
                            uv = *reinterpret_cast<const float4 *>(a.u + ((int64_t)(rb + row) * a.S + s) * d + kc + j);
                        if (tb + row < a.n)
                            xv = *reinterpret_cast<const float4 *>(a.x + (int64_t)(tb + row) * d + kc + j);
                    }
                    *reinterpret_cast<float4 *>(us + row * kRow + j) = uv;
                    *reinterpret_cast<float4 *>(xs + row * kRow + j) = xv;
                }
            } else {
                for (int e = tid; e < kTileRuns * kKC; e += 256) {
                    const int row = e / kKC, j = e % kKC;
                    float uv = 0.f, xv = 0.f;
                    if (kc + j < d) {
                        if (rb + row < a.R) uv = a.u[((int64_t)(rb + row) * a.S + s) * d + kc + j];
                        if (tb + row < a.n) xv = a.x[(int64_t)(tb + row) * d + kc + j];
                    }
                    us[row * kRow + j] = uv;
                    xs[row * kRow + j] = xv;
                }
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < kKC; kk += 8) {
                const float4 av = *reinterpret_cast<const float4 *>(ua + kk);
                const float4 bv = *reinterpret_cast<const float4 *>(xa + kk);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.x, bv.x, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.y, bv.y, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.z, bv.z, acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(av.w, bv.w, acc, 0, 0, 0);
            }
            __syncthreads();
        }

        // accumulator element v of lane l: row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32
        const int t = tb + (wave & 1) * 32 + l32;
        const int64_t ta = a.t0 + t;
        const bool mine = t < a.n && ta >= a.seg_start[s] && (s + 1 >= a.S || ta < a.seg_start[s + 1]);
        if (mine) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int run = rb + (wave >> 1) * 32 + 8 * (v / 4) + 4 * half + (v % 4);
                if (run < a.R) a.Z[(int64_t)run * a.zl.zs_r + (int64_t)a.K * a.zl.zs_i + (int64_t)t * a.zl.zs_t] = acc[v];
            }
        }
    }
}

}  // namespace

hipError_t launch_comparator_gemm(const ComparatorGemmArgs &a, hipStream_t s)
{
    if (a.n <= 0 || a.R <= 0) return hipSuccess;
    const dim3 grid((unsigned)((a.n + kTileRounds - 1) / kTileRounds), (unsigned)((a.R + kTileRuns - 1) / kTileRuns));
    if (a.vec_ok)
        hipLaunchKernelGGL(comparator_gemm_kernel<true>, grid, dim3(256), 0, s, a);
    else
        hipLaunchKernelGGL(comparator_gemm_kernel<false>, grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace oco
