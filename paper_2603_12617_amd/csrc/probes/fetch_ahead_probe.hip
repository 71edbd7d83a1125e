// Measurement probe (not part of the library): does a row that another compute unit of the same XCD has loaded
// make a later load of it fast, and does that survive updates of other rows in between -- by float atomics, or
// by plain 16-byte read-modify-writes?  Eight consumer workgroups (one per XCD) gather 2048 random rows per
// "window"; eight more fetch each window's rows ahead of them, `lag` windows at most; both sides wait for each
// other through flags with a bounded number of looks.  The sparse window kernel's fetching workgroups and its
// plain row updates rest on these figures.  Build: paper_2603_12617_amd/build.py (build_probes); run:
// _build/probes/fetch_ahead_probe.
#include <hip/hip_runtime.h>
#include <hip/amd_detail/amd_hip_unsafe_atomics.h>
#include <cstdio>
#include <cstdlib>
typedef float f4 __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("hip error %s at %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)
__device__ __forceinline__ unsigned hash(unsigned x) { x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16; return x; }

// grid 16: workgroup b < 8 consumes on XCD b (workgroups go to the XCDs in turn), workgroup 8 + b fetches for it.
// Window i = 2048 random rows.  mode 0: no fetching; 1: fetch with plain dword loads; 2: with 16-byte sc0 loads;
// 3: with sc1 loads.  atom 0: rows are only read; 1: after the gather of window i the rows of window i - 1 get a
// float atomic add each (four lanes per row); 2: a plain 16-byte read-modify-write each (a lane per row).
// Loads inside asm statements: the compiler knows nothing of them, so the registers they arrive in are named
// in the s_waitcnt statement that waits for them and stay reserved until then.
__global__ void __launch_bounds__(1024) pf(float *V, unsigned nrows, int rowfloats, int nwin, int mode, int *flags, unsigned long long *ticks, float *sink, int lag, int atom)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int x = blockIdx.x & 7;
    const float *Vb = V + x * 16;
    if (blockIdx.x >= 8) {
        if (mode == 0) return;
        for (int i = 0; i < nwin; ++i) {
            // stay at most `lag` windows ahead of the consumer
            if (threadIdx.x == 0) {
                for (int spin = 0; spin < 200000; ++spin) {
                    if (__hip_atomic_load(flags + 64 + x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= i - lag) break;
                    __builtin_amdgcn_s_sleep(8);
                }
            }
            __syncthreads();
            float g0, g1;
            f4 g4a, g4b;
            const unsigned r0 = hash((unsigned)(i * 2048 + threadIdx.x)) % nrows, r1 = hash((unsigned)(i * 2048 + 1024 + threadIdx.x)) % nrows;
            const float *p0 = Vb + (size_t)r0 * rowfloats, *p1 = Vb + (size_t)r1 * rowfloats;
            if (mode == 1) {
                asm volatile("global_load_dword %0, %1, off" : "=v"(g0) : "v"(p0) : "memory");
                asm volatile("global_load_dword %0, %1, off" : "=v"(g1) : "v"(p1) : "memory");
                asm volatile("s_waitcnt vmcnt(0)" : "+v"(g0), "+v"(g1) : : "memory");
            } else if (mode == 2) {
                asm volatile("global_load_dwordx4 %0, %1, off sc0" : "=v"(g4a) : "v"(p0) : "memory");
                asm volatile("global_load_dwordx4 %0, %1, off sc0" : "=v"(g4b) : "v"(p1) : "memory");
                asm volatile("s_waitcnt vmcnt(0)" : "+v"(g4a), "+v"(g4b) : : "memory");
            } else {
                asm volatile("global_load_dword %0, %1, off sc1" : "=v"(g0) : "v"(p0) : "memory");
                asm volatile("global_load_dword %0, %1, off sc1" : "=v"(g1) : "v"(p1) : "memory");
                asm volatile("s_waitcnt vmcnt(0)" : "+v"(g0), "+v"(g1) : : "memory");
            }
            __syncthreads();
            if (threadIdx.x == 0) __hip_atomic_store(flags + x, i + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        return;
    }
    float acc = 0.f;
    unsigned long long t_sum = 0, u_sum = 0;
    for (int i = 0; i < nwin; ++i) {
        if (threadIdx.x == 0) {
            __hip_atomic_store(flags + 64 + x, i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (mode != 0)
                for (int spin = 0; spin < 200000; ++spin) {
                    if (__hip_atomic_load(flags + x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) > i) break;
                    __builtin_amdgcn_s_sleep(8);
                }
        }
        __syncthreads();
        const unsigned long long t0 = wall_clock64();
        f4 a, b;
        const unsigned r0 = hash((unsigned)(i * 2048 + threadIdx.x)) % nrows, r1 = hash((unsigned)(i * 2048 + 1024 + threadIdx.x)) % nrows;
        const float *p0 = Vb + (size_t)r0 * rowfloats, *p1 = Vb + (size_t)r1 * rowfloats;
        asm volatile("global_load_dwordx4 %0, %1, off sc0" : "=v"(a) : "v"(p0) : "memory");
        asm volatile("global_load_dwordx4 %0, %1, off sc0" : "=v"(b) : "v"(p1) : "memory");
        asm volatile("s_waitcnt vmcnt(0)" : "+v"(a), "+v"(b) : : "memory");
        acc += a[0] + b[1];
        __syncthreads();
        if (threadIdx.x == 0) t_sum += wall_clock64() - t0;
        const unsigned long long t1 = wall_clock64();
        if (atom == 2 && i > 0) {
            // plain read-modify-write of the rows of window i - 1, a lane per row
            f4 m0, m1;
            const unsigned q0 = hash((unsigned)((i - 1) * 2048 + threadIdx.x)) % nrows, q1 = hash((unsigned)((i - 1) * 2048 + 1024 + threadIdx.x)) % nrows;
            float *w0 = const_cast<float *>(Vb) + (size_t)q0 * rowfloats, *w1 = const_cast<float *>(Vb) + (size_t)q1 * rowfloats;
            asm volatile("global_load_dwordx4 %0, %1, off sc0" : "=v"(m0) : "v"(w0) : "memory");
            asm volatile("global_load_dwordx4 %0, %1, off sc0" : "=v"(m1) : "v"(w1) : "memory");
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(m0), "+v"(m1) : : "memory");
            m0 += 1.0f; m1 += 1.0f;
            *reinterpret_cast<f4 *>(w0) = m0;
            *reinterpret_cast<f4 *>(w1) = m1;
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }
        if (atom == 1 && i > 0) {
            for (int k = 0; k < 8; ++k) {
                const unsigned rr = hash((unsigned)((i - 1) * 2048 + (k * 16 + wave) * 16 + (lane >> 2))) % nrows;
                unsafeAtomicAdd(const_cast<float *>(Vb) + (size_t)rr * rowfloats + (lane & 3), 1.0f);
            }
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
        }
        if (threadIdx.x == 0) u_sum += wall_clock64() - t1;
    }
    if (threadIdx.x == 0) { ticks[x] = t_sum; ticks[8 + x] = u_sum; }
    if (acc == 12345.f) sink[threadIdx.x] = acc;
}

int main()
{
    const size_t total = (size_t)640 << 20;
    float *V, *sink; int *flags; unsigned long long *ticks;
    CK(hipMalloc(&V, total)); CK(hipMemset(V, 0, total)); CK(hipMalloc(&sink, 4096));
    CK(hipMalloc(&flags, 1024)); CK(hipMalloc(&ticks, 128));
    const int rowfloats = 160, nwin = 512;
    const unsigned nrows = (unsigned)(total / (rowfloats * 4));
    for (int atom = 0; atom < 3; ++atom)
    for (int mode = 0; mode < 2; ++mode)
        for (int lag : {1, 4}) {
            CK(hipMemset(flags, 0, 1024));
            hipLaunchKernelGGL(pf, dim3(16), dim3(1024), 0, 0, V, nrows, rowfloats, nwin, mode, flags, ticks, sink, lag, atom);
            CK(hipDeviceSynchronize());
            unsigned long long h[16]; CK(hipMemcpy(h, ticks, 128, hipMemcpyDeviceToHost));
            printf("update %s, fetch ahead %s, lag %d: gather of 2048 rows, us per window on XCD 0..7:", atom == 0 ? "none" : (atom == 1 ? "atomics" : "read-modify-write"), mode ? "yes" : "no", lag);
            for (int i = 0; i < 8; ++i) printf(" %.2f", h[i] / 100.0 / nwin);
            printf("  | the updates:");
            for (int i = 0; i < 8; i += 4) printf(" %.2f", h[8 + i] / 100.0 / nwin);
            printf("\n"); fflush(stdout);
        }
    return 0;
}
