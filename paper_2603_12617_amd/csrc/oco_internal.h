// Internal declarations shared by the translation units of liboco (host API,
// dense-round kernel, sparse-round kernel, meta/finalize kernels).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace oco {

constexpr int kWave = 64;          // gfx950 wavefront width
constexpr float kFoldLo = 0x1p-24f; // lazy scale is folded into the vector outside [lo, hi]
constexpr float kFoldHi = 0x1p+24f;

// Z holds, for the rounds of one oco_run_rounds call, the prediction
// z_t^i = <w_t^i, x_t> of every base learner (i < K) and of the comparator
// (i == K).  Element (r, i, t) lives at Z[r*zs_r + i*zs_i + t*zs_t].
struct ZLayout {
    int64_t zs_r, zs_i, zs_t;
};

// Tuning choices of a state (oco_set_option), indexed by oco_option; -1 = the library decides.
constexpr int kNumOptions = 12;
struct Tuning {
    int64_t v[kNumOptions];
    __host__ Tuning() { for (auto &e : v) e = -1; }
    int64_t get(int key) const { return v[key]; }
};

// How the dense round kernel of a state is launched: depends on the configuration and the
// tuning choices only (not on n or t0), so it is worked out once and kept in the state.
struct DensePlanCache {
    bool valid = false;
    const void *kern = nullptr;
    size_t smem = 0;
    int wpb = 0;
    int64_t nwg = 0, batches = 0;
    int per_run = 0;
};

// Called after the round kernel of every piece of a call has been enqueued: rounds
// [off, off + len) of the call have their predictions in Z once that kernel finishes.
struct PieceHook {
    hipError_t (*fn)(void *ctx, int off, int len);
    void *ctx;
    // Optional: a stream for work of the call that the round kernels neither wait for nor feed
    // (it starts after the work already on the call's stream, and what fn enqueues follows it).
    hipError_t (*beside)(void *ctx, hipStream_t *out) = nullptr;
    // Optional, with `beside`: mark remembers what is on that stream now; after wait_mark the call's stream
    // goes on only when that work is done (for work beside the round kernels that a later one of them needs).
    hipError_t (*mark)(void *ctx) = nullptr;
    hipError_t (*wait_mark)(void *ctx) = nullptr;
};

// Event pairs around the launches of a call's dominant kernel (benchmarks: the duration of that
// kernel alone, launch by launch).  The launchers call begin / end around each such launch; with
// no clock, or past its capacity, they cost nothing and only count.
struct LaunchClock {
    static constexpr int kPairs = 64;
    hipEvent_t ev[2 * kPairs] = {};
    int launches = 0;          // of the last call
    int timed = 0;             // of those, how many have an event pair
    const char *kernel = "";   // which kernel the launcher timed
    hipError_t begin(hipStream_t s) { return timed < kPairs && ev[2 * timed] ? hipEventRecord(ev[2 * timed], s) : hipSuccess; }
    hipError_t end(hipStream_t s)
    {
        ++launches;
        if (timed >= kPairs || !ev[2 * timed + 1]) return hipSuccess;
        return hipEventRecord(ev[2 * timed++ + 1], s);
    }
};
inline hipError_t clock_begin(LaunchClock *c, hipStream_t s, const char *kernel)
{
    if (!c) return hipSuccess;
    c->kernel = kernel;
    return c->begin(s);
}
inline hipError_t clock_end(LaunchClock *c, hipStream_t s) { return c ? c->end(s) : hipSuccess; }

// ---- dense rounds -----------------------------------------------------------
struct DenseArgs {
    const float *x;          // round stream (or gradient stream for the linear loss)
    int64_t x_run_stride;    // elements between runs (unused when x_shared)
    const float *y;          // labels, may be null (linear loss)
    int64_t y_run_stride;
    const float *u;          // comparator segments [R][S][d]
    const int64_t *seg_start;// device copy, [S]
    int S;
    float *V;                // [R][K][d]  iterate = sigma * V
    float *sigma;            // [R][K]
    double *n2;              // [R][K]  ||V row||^2
    float *x2;               // scratch: ||x_t||^2 per round of this call, [n] or [R][x2_run_stride]
    int64_t x2_run_stride;
    const float *eta;        // [K]
    float *Z;
    ZLayout zl;
    int d, K, R;
    int64_t t0;              // absolute index of the first round of this call
    int n;                   // rounds in this call
    float D;
    int x_shared;
    int vec_ok;              // rows of x are 16-byte aligned and d % 4 == 0
    int per_run;             // wavefront tasks per run: K + 1 with the comparator's, K when its
                             // predictions come from the contraction kernel (set by the launcher)
    // optimistic two-step update (Eq. (3)); V then holds the intermediate model w^
    int optimistic;
    float *ha;               // [R][K]  eta_i c_{t-1}^i: the hint is ha * x_{t-1}
    float *hp;               // [R][K]  <w^_t, x_{t-1}>
    float *g01;              // scratch like x2: <x_{t-1}, x_t> per round of this call
    float *xlast;            // [1 or R][d]  last round row of the previous call (0 before round 0)
    float *x2last;           // [1 or R]     its squared norm
    const Tuning *tune;      // never null
    LaunchClock *clock;      // null unless the call is timed
    DensePlanCache *plan;    // never null
    float *gram;             // shared streams: dense_gram_bytes(n_max, d) of scratch for the windowed path
    int64_t n_max;           // the state's largest call (lays that scratch out)
};
hipError_t launch_dense_rounds(const DenseArgs &a, int loss, hipStream_t s, const PieceHook *hook);
// the windowed path (dense_window.hip): whether a configuration takes it, and its launcher
bool dense_window_wanted(const DenseArgs &a);
hipError_t launch_dense_window(const DenseArgs &a, int loss, hipStream_t s, const PieceHook *hook);
hipError_t launch_hint_scalars(const DenseArgs &a, hipStream_t s);
hipError_t launch_keep_last_row(const DenseArgs &a, hipStream_t s);
size_t dense_gram_bytes(int64_t n_max, int64_t d);

// comparator predictions of a shared dense stream as one contraction (rows K of Z)
struct ComparatorGemmArgs {
    const float *x;          // [n][d]
    const float *u;          // [R][S][d]
    const int64_t *seg_start;// device, [S]
    int S;
    float *Z;
    ZLayout zl;
    int d, K, R;
    int64_t t0;
    int n;
    int vec_ok;              // rows of x and u are 16-byte aligned and d % 4 == 0
};
hipError_t launch_comparator_gemm(const ComparatorGemmArgs &a, hipStream_t s);
bool dense_supported(int64_t d, int x_shared);

// ---- sparse rounds ----------------------------------------------------------
struct SparseArgs {
    const int32_t *col;      // [n][nnz]
    const float *val;        // [n][nnz]
    const float *y;
    int64_t y_run_stride;
    const float *u;          // [R][S][d]
    const int64_t *seg_start;
    int S;
    float *V;                // [d][RKp]: coordinate-major, the R*K learners interleaved (RKp: padded row length)
    double *sigma;           // [RKp]
    double *n2;              // [RKp]  ||V column||^2
    const float *eta;        // [K]
    float *Z;
    ZLayout zl;
    int d, K, R, nnz, RKp;
    int64_t t0;
    int n;
    double D;
    void *scratch;           // sparse_scratch_bytes(n_max) bytes: per-window Gram data of the call
    // optimistic two-step update (Eq. (3)); V then holds the intermediate model w^
    int optimistic;
    float *ha;               // [RKp]  eta_i c_{t-1}^i: the hint is ha * x_{t-1}
    float *hp;               // [RKp]  <w^_t, x_{t-1}>
    float *hx;               // [RKp]  ||x_{t-1}||^2 (the same for all learners; kept per lane)
    int32_t *last_col;       // [OCO_MAX_NNZ]  last round row of the previous call (zeros before round 0)
    float *last_val;         // [OCO_MAX_NNZ]
    float *xlast_dense;      // [d]  the same row scattered into a dense vector (for the export)
    const Tuning *tune;      // never null
    LaunchClock *clock;      // null unless the call is timed
};
hipError_t launch_sparse_rounds(const SparseArgs &a, int loss, hipStream_t s, const PieceHook *hook);
size_t sparse_scratch_bytes(int64_t n_max);

// ---- meta learner + regret --------------------------------------------------
struct MetaArgs {
    const float *Z;
    ZLayout zl;
    const float *y;
    int64_t y_run_stride;
    double *L;               // [R][K] cumulative losses, updated in place
    double *last;            // [R][K] last observed losses (the meta learner's hint), updated in place; or null
    double *regret;          // [R]
    double eps;
    int K, R, n;
};
hipError_t launch_meta(const MetaArgs &a, int loss, hipStream_t s);

// ---- state export -----------------------------------------------------------
struct ExportArgs {
    const float *V;
    const void *sigma;       // float [R][K] (dense) or double [RKp] (sparse)
    const double *L;
    const double *last;      // the meta learner's hint, or null
    double eps;
    float *W, *p, *wbar;     // any may be null
    int d, K, R, RKp;
    int sparse;
    // optimistic: the exported iterate is Proj[sigma V - ha xlast].  Dense: xlast [1 or R][d],
    // x2last [1 or R].  Sparse: xlast [d] (dense copy of the last sparse row), x2last [RKp].
    int optimistic;
    const float *ha, *hp, *xlast, *x2last;
    const double *n2;
    int x_shared;
    float D;
};
hipError_t launch_export(const ExportArgs &a, hipStream_t s);
hipError_t launch_accel_bounds(const double *regret, int R, int64_t t, int64_t k, double alpha, double *out,
                               hipStream_t s);

// step sizes as a kernel argument
struct EtaTable { float v[64]; };
hipError_t launch_set_eta(float *eta_dev, const EtaTable &tab, int K, hipStream_t s);

// fills `bytes` (a multiple of 16) of device memory with zero using a kernel,
// and sets every sigma to 1
hipError_t launch_init_state(void *zero_base, size_t zero_bytes, void *sigma, int64_t n_sigma,
                             int sigma_is_double, hipStream_t s);

}  // namespace oco
