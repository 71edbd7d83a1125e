/*
 * liboco -- batched simulation of the online-ensemble learner on one MI355X.
 *
 * The library advances R independent runs of the learner of Sec. 3.3: K
 * projected online-gradient-descent base learners (Sec. 3.1 update on the
 * domain of Assumption 2, an L2 ball of radius D), a Hedge meta learner over
 * their cumulative losses, and the dynamic regret of Eq. (2) against a
 * piecewise-constant comparator sequence.  Losses are generalised linear,
 * f_t(w) = phi(<w, x_t>; y_t), so grad f_t(w) = phi'(<w, x_t>; y_t) x_t.
 *
 * Per run and round t (0-based here; the paper's round t+1), with
 * L_t^i = sum_{s<t} f_s(w_s^i):
 *     p_t^i      = exp(-eps L_t^i) / sum_j exp(-eps L_t^j)           (Hedge)
 *     w_t        = sum_i p_t^i w_t^i                                 (combined iterate)
 *     regret    += f_t(w_t) - f_t(u_t)                               (Eq. (2))
 *     w_{t+1}^i  = Proj_{||w||<=D}[ w_t^i - eta_i grad f_t(w_t^i) ]  (each learner at its own iterate)
 * starting from w_0^i = 0, L_0 = 0, regret = 0.
 *
 * Conventions
 *  - Every function returns OCO_OK (0) or a negative oco_status; nothing
 *    throws or aborts.  All argument checks happen on the host before any
 *    kernel is launched.
 *  - "host" / "device" is stated for every pointer.  The library allocates no
 *    device memory: the caller provides one workspace (oco_workspace_bytes)
 *    and owns every input and output buffer.  Device pointers to float32 /
 *    int32 data must be 4-byte aligned (OCO_EINVAL otherwise); round streams
 *    whose rows are 16-byte aligned (pointer and run stride multiples of 16 bytes,
 *    d a multiple of 4) take the kernels' vector-load path, others a slower
 *    scalar one with the same results.  The comparator array must be 16-byte
 *    aligned, float64 outputs 8-byte, the workspace 256-byte aligned.
 *  - A HIP error in the middle of oco_run_rounds (after part of the call's work
 *    was enqueued) leaves the device state undefined: the state is marked failed
 *    and every later call on it returns OCO_EHIP until oco_reset.
 *  - All GPU work is ordered on the HIP stream given to oco_create: a call may run
 *    part of its work on a second stream of the library's own, which starts after
 *    the work already on the caller's stream and which the caller's stream waits
 *    for before the call's work counts as done.  Input buffers are borrowed until
 *    that work has finished.
 *  - Results are a pure function of (config, options, inputs, call boundaries).
 *    Dense configurations on the register kernel: splitting [0, T) into
 *    oco_run_rounds calls in any way gives bit-identical state and regret; on the
 *    windowed kernel (OCO_OPT_DENSE_PATH) the rounds are worked in windows of 64
 *    whose inner products are grouped differently at the start of a call than
 *    inside it: the same calls give the same bits, different splits agree to
 *    float32 rounding.  Sparse configurations work in segments of 4096 rounds of
 *    the horizon: splits at multiples of 4096 are bit-identical, other splits
 *    regroup float32 sums and agree to rounding.
 *  - Arithmetic: iterates, inner products and the projection in float32;
 *    losses, cumulative losses, Hedge weights and regret in float64.
 */
#ifndef OCO_H
#define OCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct oco_state oco_state; /* opaque host object */

typedef enum {
    OCO_OK = 0,
    OCO_EINVAL = -1,  /* NULL pointer, non-positive size, non-finite parameter, misaligned buffer */
    OCO_ESEQ = -2,    /* t0 is not the number of rounds already consumed */
    OCO_ERANGE = -3,  /* t0 + n exceeds T, n exceeds n_max, or too many comparator segments */
    OCO_ENOMEM = -4,  /* workspace smaller than oco_workspace_bytes */
    OCO_EHIP = -5,    /* a HIP runtime call failed (no usable device, launch error) */
    OCO_ENOCOMP = -6, /* oco_run_rounds before oco_set_comparator */
    OCO_EUNSUPPORTED = -7 /* shape outside what the kernels cover (see oco_config) */
} oco_status;

typedef enum {
    OCO_LINEAR = 0,   /* phi(z; y) = z            (x_t is the gradient g_t, y unused) */
    OCO_SQUARED = 1,  /* phi(z; y) = (z - y)^2     gradient 2 (z - y) x_t             */
    OCO_LOGISTIC = 2  /* phi(z; y) = log(1 + exp(-y z)), y in {-1, +1}                */
} oco_loss;

#define OCO_MAX_SEGMENTS 4096   /* comparator segments per run */
#define OCO_MAX_K 64            /* base learners per run */
#define OCO_MAX_DENSE_D 65536   /* dense rounds: per-run streams need d <= 4096 (the iterate lives in one
                                   wavefront's registers); a shared stream may go up to this (iterates in
                                   registers up to 4096, beyond that streamed from HBM once per 64 rounds) */
#define OCO_MAX_NNZ 64          /* entries per sparse round */

typedef struct {
    int64_t d;            /* dimension of w; dense rounds: see OCO_MAX_DENSE_D        */
    int64_t K;            /* base learners per run (the paper's N), 1..OCO_MAX_K      */
    int64_t T;            /* horizon: total rounds                                    */
    int64_t R;            /* independent runs                                         */
    double D;             /* radius of the domain { ||w||_2 <= D } (Assumption 2)     */
    double G;             /* gradient-norm bound of Assumption 2; informational --
                             it enters only through the step grid                     */
    const double *eta;    /* host, [K]: step sizes (see oco_step_grid); copied        */
    double eps;           /* meta learning rate of Hedge, >= 0                        */
    int32_t loss;         /* oco_loss                                                 */
    int32_t x_shared;     /* 1: one round stream for all runs; 0: one per run
                             (dense only; sparse streams are always shared)           */
    int32_t sparse_nnz;   /* 0: dense rounds; >0: every round has exactly this many
                             (column, value) entries, columns distinct within a round */
    int32_t optimistic;   /* 0: plain update w_{t+1} = Proj[w_t - eta grad f_t(w_t)] (Sec. 3.1);
                             1: optimistic two-step update of Eq. (3) with the last round's
                             gradient as hint (Sec. 3.2), every base learner on its own:
                               w_t = Proj[w^_t - eta h_t],  w^_{t+1} = Proj[w^_t - eta grad f_t(w_t)],
                               h_{t+1} = grad f_t(w_t),  h_1 = 0,  w^_1 = 0.
                             Predictions, losses and regret are those of the played iterates
                             w_t; oco_get_state returns the iterates that would be played
                             next.  K = 1 is the paper's method; for K > 1 Hedge weighs the
                             played iterates (not analysed in the paper);
                             2: optimism at both levels of the ensemble (appendix on combining
                             optimistic and ensemble learning, which names the combination and
                             gives no update rule).  Reading built here: base learners as 1;
                             the meta learner is Hedge on the cumulative losses plus a hint for
                             the coming loss, p_t^i ~ exp(-eps (L_{t-1}^i + m_t^i)), with the
                             last observed loss as hint, m_t^i = f_{t-1}(w_{t-1}^i), m_1 = 0;
                             no correction term.  oco_get_state hands back the weights of
                             round T + 1                                                  */
    int64_t n_max;        /* largest n of any oco_run_rounds call; 0 means T          */
} oco_config;

typedef struct {
    /* all device pointers, read-only, indexed by the round RELATIVE to t0 */
    const float *x;       /* dense: [n][d] if x_shared, else run r at x + r*x_run_stride;
                             for OCO_LINEAR this is the gradient stream g              */
    const int32_t *col;   /* sparse: [n][nnz] column indices in [0, d)                 */
    const float *val;     /* sparse: [n][nnz] values                                   */
    const float *y;       /* run r at y + r*y_run_stride, [n] each; NULL for OCO_LINEAR */
    int64_t x_run_stride; /* elements between runs of x; 0 means n*d                   */
    int64_t y_run_stride; /* elements between runs of y; 0 means n                     */
} oco_rounds;

/* Step grid of the proof of Corollary 3: eta_i = 2^i D / (G sqrt(T)), i = 0..K-1
 * (the paper indexes it i-1, i = 1..N).  out: host [K]. */
int oco_step_grid(double D, double G, int64_t T, int64_t K, double *out);

/* Number of base learners the proof of Corollary 3 prescribes: ceil(log2(1+T)/2) + 1. */
int64_t oco_paper_num_learners(int64_t T);

/* Bytes of device workspace oco_create needs for this config; 0 if the config is invalid
 * or unsupported. */
size_t oco_workspace_bytes(const oco_config *cfg);

/* Validates cfg, lays the state out in the caller's device workspace and zeroes it
 * (w_0 = 0, L_0 = 0, regret = 0) on `hip_stream` (a hipStream_t, NULL = default stream).
 * dev_ws: device, >= oco_workspace_bytes(cfg) bytes, owned by the caller and borrowed until
 * oco_destroy.  *out receives a host object to release with oco_destroy. */
int oco_create(const oco_config *cfg, void *dev_ws, size_t ws_bytes, void *hip_stream,
               oco_state **out);

/* The same as oco_create for callers that cannot provide (or allocate) a workspace: code that
 * runs where hipMalloc is not allowed -- under HIP graph capture, inside a serving loop, in a
 * harness that forbids allocation.  The state, the predictions of a call and the kernels'
 * scratch live in a device array of OCO_STATIC_WS_BYTES that is part of the library's image
 * (one copy per GPU, held until the process ends); a configuration whose oco_workspace_bytes
 * exceeds that returns OCO_ENOMEM (lower n_max to make it fit).  The call allocates no device
 * memory, creates no stream or event (work of a call that could run beside the round kernels
 * stays in line, and oco_set_timing is refused with OCO_EUNSUPPORTED) and touches the device
 * only with the kernel that zeroes the state.  Inputs and outputs stay the caller's, as in
 * every other call.  All states created this way on one GPU share the one array: a second
 * oco_create_static (or oco_reset) overwrites the first state's memory, and calls on two such
 * states that overlap in time race.  Results are identical to those of oco_create. */
#define OCO_STATIC_WS_BYTES (64u << 20)
int oco_create_static(const oco_config *cfg, void *hip_stream, oco_state **out);

/* Tuning choices of a state: which of several equivalent kernels or launch shapes a call uses.
 * value -1 (the default of every key) leaves the choice to the library.  Results agree with the
 * reference to the stated tolerances under every choice; choices that change how float32 sums
 * are grouped are marked (~).  OCO_EINVAL for an unknown key or a value the key does not take. */
typedef enum {
    OCO_OPT_META_BESIDE = 0,     /* 0: meta kernel after the round kernels, on the call's stream;
                                    1: beside them on the library's second stream where the launcher allows */
    OCO_OPT_DENSE_PATH = 1,      /* (~) 1: one wavefront per learner, iterate in registers;
                                    2: windows of 64 rounds as contractions on the matrix cores (shared stream) */
    OCO_OPT_DENSE_WPB = 2,       /* wavefronts per workgroup of the register kernel */
    OCO_OPT_COMPARATOR_GEMM = 3, /* (~) comparator predictions of a shared stream: 0 in the round kernel, 1 as a contraction */
    OCO_OPT_DENSE_HALF = 4,      /* (~) 1: two learners per wavefront (shared stream, d <= 1024); 0: never */
    OCO_OPT_DENSE_PIECES = 5,    /* launches a dense call is cut into */
    OCO_OPT_SPARSE_LPW = 6,      /* (~) learners per workgroup of the sparse kernel: 4, 8, 16, 32, 64 */
    OCO_OPT_SPARSE_PIPE = 7,     /* (~) 0: sparse windows one after the other, no pipeline */
    OCO_OPT_VERBOSE = 8,         /* 1: launch plans on stderr */
    OCO_OPT_WINDOW_RESIDENT = 9, /* (~) windowed dense path, where the iterates live between windows:
                                    0: HBM, two tiles of 16 learners per workgroup; 1: registers of the
                                    workgroup (d <= 4096, else as 0); 2: HBM, one tile, 16 wavefronts;
                                    3: HBM, four tiles, operands brought to LDS by loading wavefronts;
                                    4: registers, two tiles per workgroup (d <= 1024, else as 0)
                                    (with the optimistic update 1 and 2 are taken as 0) */
    OCO_OPT_SPARSE_FETCH = 10,   /* 0: no workgroups that fetch the rows of coming sparse windows into L2 ahead of
                                    the working ones (the library adds them where the grid leaves most of the chip idle) */
    OCO_OPT_COUNT = 11
} oco_option;
int oco_set_option(oco_state *st, int key, int64_t value);

/* Comparator sequence of Eq. (2): u_dev device [R][S][d] float32 (borrowed until the last
 * oco_run_rounds has finished), segment s of every run is active for rounds
 * seg_start[s] <= t < seg_start[s+1] (last segment to T).  seg_start: host [S], copied,
 * strictly increasing with seg_start[0] == 0; 1 <= S <= OCO_MAX_SEGMENTS. */
int oco_set_comparator(oco_state *st, const float *u_dev, const int64_t *seg_start_host,
                       int64_t S);

/* Advances every run by rounds t0 .. t0+n-1.  t0 must equal the rounds consumed so far
 * (OCO_ESEQ), t0 + n <= T and n <= n_max (OCO_ERANGE).  n == 0 is a no-op.  Asynchronous:
 * returns after enqueueing on the stream. */
int oco_run_rounds(oco_state *st, const oco_rounds *rounds, int64_t t0, int64_t n);

/* Dynamic regret of every run over the rounds consumed so far.  out_host: host [R].
 * Synchronises the stream. */
int oco_regret(oco_state *st, double *out_host);

/* Writes the current iterates w^i (W_dev: device [R][K][d]), the Hedge weights for the next
 * round (p_dev: device [R][K]) and the combined iterate sum_i p^i w^i (wbar_dev: device
 * [R][d]); any of the three may be NULL.  Asynchronous on the stream. */
int oco_get_state(oco_state *st, float *W_dev, float *p_dev, float *wbar_dev);

/* Accepted-length and acceleration-rate bounds of Lemma 1 and Theorem 1 for every run, from
 * its dynamic regret Reg over the t rounds consumed so far, the candidate length k >= 1 and
 * the draft/target inference-time ratio alpha >= 0:
 *   out[r][0] = (k+1) t / (1 + (k+1) sqrt(Reg / (2 t)))     lower bound on the expected length
 *   out[r][1] = (k+1) t                                      upper bound
 *   out[r][2] = out[r][0] / (t (alpha k + 1))                lower bound on the rate gamma
 *   out[r][3] = (k+1) / (alpha k + 1)                        upper bound
 * A negative regret (possible against an arbitrary comparator; the lemma's regret is a sum of
 * KL terms) is taken as 0.  out_dev: device [R][4] float64, caller-owned.  OCO_ESEQ before the
 * first round.  Asynchronous on the stream. */
int oco_accel_bounds(oco_state *st, int64_t k, double alpha, double *out_dev);

/* Cumulative base-learner losses L^i over the rounds consumed so far.  out_host: host [R][K].
 * Synchronises the stream. */
int oco_cum_losses(oco_state *st, double *out_host);

/* Back to round 0 (w = 0, L = 0, regret = 0); keeps the comparator and the options, clears a
 * failed mark.  Asynchronous. */
int oco_reset(oco_state *st);

/* Kernel timing for benchmarks.  After oco_set_timing(st, 1) every oco_run_rounds call records
 * HIP events on the state's stream; oco_last_timing waits for the most recent call's events and
 * writes two durations in milliseconds to ms_host: host [2],
 * [0] = the round kernels of the call (steps S0-S2, S4 of a round: stream x, predict, slope, step,
 *       project; a long call goes to the GPU as several launches),
 * [1] = from their end to the end of the call: the meta kernel (Hedge weights, losses, regret),
 *       or, where the meta kernel of each piece of the call already ran beside the round kernels
 *       of the next piece on a second stream, the part of it that was left.
 * Timing changes nothing in what is enqueued.  OCO_EINVAL if timing is off or no call has been
 * made since it was switched on. */
int oco_set_timing(oco_state *st, int enable);
int oco_last_timing(oco_state *st, float *ms_host);

/* The dominant kernel of the most recent timed call alone, launch by launch: the kernel that
 * works the rounds (Sec. 3.1 / 3.3 update of the base learners), without the passes that prepare
 * its inputs or the meta kernel.  *ms_sum_host = summed duration of the launches that were timed
 * (event pairs on the state's stream), *timed_host = how many those were (at most 64 per call),
 * *launches_host = launches of that kernel in the call, *kernel (may be null) = its name, a
 * static string.  Same preconditions and errors as oco_last_timing. */
int oco_last_kernel_timing(oco_state *st, float *ms_sum_host, int *timed_host, int *launches_host, const char **kernel);

/* Rounds consumed so far, or a negative oco_status. */
int64_t oco_rounds_done(const oco_state *st);

/* Releases the host object (the device workspace stays the caller's).  NULL is allowed. */
void oco_destroy(oco_state *st);

/* Static, human-readable text for a status code. */
const char *oco_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* OCO_H */
