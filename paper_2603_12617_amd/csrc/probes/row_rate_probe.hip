// Measurement probe (not part of the library): how fast one workgroup of 16 wavefronts is served random
// 16-byte pieces of 640-byte rows -- the access pattern of the sparse rounds (a workgroup owns four learners
// of a coordinate-major iterate) -- as a function of the span the rows are drawn from (HBM, the memory-side
// cache, L2), for 16-byte loads by one lane per row, 4-byte loads by four lanes per row, and float atomics.
// The sparse window kernel's choices (a lane per row, workgroups that fetch rows into L2 ahead) rest on
// these figures.  Build: paper_2603_12617_amd/build.py (build_probes); run: _build/probes/row_rate_probe.
#include <hip/hip_runtime.h>
#include <hip/amd_detail/amd_hip_unsafe_atomics.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
typedef float f4 __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("hip error %s at %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)

__device__ __forceinline__ unsigned hash(unsigned x) { x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16; return x; }

// mode 0: x4 sc0 loads, a lane per row; mode 1: dword sc0 loads, 4 lanes per row; mode 2: float atomics, 4 lanes per row
// mode 3: x4 plain loads
template <int MODE>
__global__ void __launch_bounds__(1024) probe(float *V, unsigned nrows, int rowfloats, int iters, float *sink, int sorted)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const float *Vb = V + blockIdx.x * 4;
    float acc = 0.f;
    for (int it = 0; it < iters; ++it) {
        f4 r[3];
        float s[3];
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const unsigned key = (unsigned)((it * 3 + u) * 16 + wave);
            unsigned row;
            if (MODE == 0 || MODE == 3) row = hash(key * 64u + lane) % nrows;
            else row = hash(key * 16u + (lane >> 2)) % nrows;
            if (sorted) {   // rows of one instruction ascend through a 1/16 share of the rows per wavefront
                const unsigned per = nrows / 16;
                const unsigned slot = (MODE == 0 || MODE == 3) ? lane : (lane >> 2);
                const unsigned nsl = (MODE == 0 || MODE == 3) ? 64 : 16;
                row = wave * per + slot * (per / nsl) + hash(key) % (per / nsl);
            }
            const float *p = Vb + (size_t)row * rowfloats;
            if (MODE == 0) asm volatile("global_load_dwordx4 %0, %1, off sc0" : "=v"(r[u]) : "v"(p) : "memory");
            if (MODE == 3) r[u] = *reinterpret_cast<const f4 *>(p);
            if (MODE == 1) s[u] = __hip_atomic_load(p + (lane & 3), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            if (MODE == 2) unsafeAtomicAdd(const_cast<float *>(p) + (lane & 3), 1.0f);
        }
        if (MODE == 0) asm volatile("s_waitcnt vmcnt(0)" : "+v"(r[0]), "+v"(r[1]), "+v"(r[2]) : : "memory");
        if (MODE == 0 || MODE == 3) acc += r[0][0] + r[1][1] + r[2][2];
        if (MODE == 1) acc += s[0] + s[1] + s[2];
    }
    if (MODE == 2) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    if (acc == 12345.f) sink[threadIdx.x] = acc;
}

template <int MODE> void run(const char *name, float *V, size_t bytes, int rowfloats, int grid, float *sink, int sorted)
{
    const unsigned nrows = (unsigned)(bytes / (rowfloats * 4));
    const int iters = 2000;
    hipEvent_t e0, e1;
    CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
    hipLaunchKernelGGL(probe<MODE>, dim3(grid), dim3(1024), 0, 0, V, nrows, rowfloats, 200, sink, sorted);
    CK(hipDeviceSynchronize());
    CK(hipEventRecord(e0));
    hipLaunchKernelGGL(probe<MODE>, dim3(grid), dim3(1024), 0, 0, V, nrows, rowfloats, iters, sink, sorted);
    CK(hipEventRecord(e1));
    CK(hipDeviceSynchronize());
    float ms; CK(hipEventElapsedTime(&ms, e0, e1));
    const double rows_per_wg = (double)iters * 3 * 16 * ((MODE == 0 || MODE == 3) ? 64 : 16);
    printf("%-28s span %7.1f MB grid %3d sorted %d: %.3f ms, %.2f ns per row per workgroup (%.2f clk at 2.4 GHz)\n", name, bytes / 1048576.0, grid,
           sorted, ms, ms * 1e6 / rows_per_wg, ms * 1e6 / rows_per_wg * 2.4);
    fflush(stdout);
}

int main()
{
    const size_t total = (size_t)640 << 20;
    float *V, *sink;
    CK(hipMalloc(&V, total)); CK(hipMemset(V, 0, total)); CK(hipMalloc(&sink, 4096));
    const int rowfloats = 160;    // 640-byte rows as for 128 learners with padding (an odd number of 128-byte lines)
    for (int grid : {1, 32}) {
        for (size_t span : {(size_t)640 << 20, (size_t)64 << 20, (size_t)2 << 20, (size_t)64 << 10}) {
            run<0>("x4 sc0, lane per row", V, span, rowfloats, grid, sink, 0);
            run<3>("x4 plain, lane per row", V, span, rowfloats, grid, sink, 0);
            run<1>("dword sc0, 4 lanes per row", V, span, rowfloats, grid, sink, 0);
            run<2>("atomic add, 4 lanes per row", V, span, rowfloats, grid, sink, 0);
        }
        run<0>("x4 sc0, lane per row", V, total, rowfloats, grid, sink, 1);
        run<2>("atomic add, 4 lanes per row", V, total, rowfloats, grid, sink, 1);
    }
    return 0;
}
