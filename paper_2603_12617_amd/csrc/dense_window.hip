// Dense rounds of the base learners on a shared round stream, worked in windows of 64 rounds as
// contractions on the matrix cores (Sec. 3.1 update inside the ensemble of Sec. 3.3).
//
// The update of a base learner, w_{t+1} = Proj[w_t - eta c_t x_t] with c_t = phi'(<w_t, x_t>; y_t),
// keeps the iterate in the span of the window's start w_s and the window's round rows, whatever
// the projections do (a projection onto the ball only rescales):
//     w_t = A_t w_s - sum_{s <= r < t} a_r rho_{r,t} x_r,   a_r = eta c_r,
//     rho_{r,t} = f_r f_{r+1} ... f_{t-1},   A_t = f_s ... f_{t-1},   f_r = min(1, D / ||w_r - a_r x_r||).
// So for a window of B = 64 rounds and a tile of M = 16 learners (any 16 learners: the stream is
// shared), with W the M x d matrix of iterates and X_w the B x d block of round rows:
//   (1) Q0 = W X_w^T                                  (M x B contraction over d, matrix cores)
//   (2) the 64 dependent rounds on scalars only: with G = X_w X_w^T (once per window for all
//       learners, pre-pass), p_{t2} = <w_t, x_{t2}> for the rounds t2 >= t still to come obeys
//           p_{t2} <- f_t (p_{t2} - a_t G[t][t2]),
//       the prediction of round t is p_t itself, and the squared norm follows from
//           ||w_t - a_t x_t||^2 = ||w_t||^2 - 2 a_t <w_t, x_t> + a_t^2 G[t][t]
//       (float64 scalars; one wavefront, a quad of lanes per learner, each lane of the quad
//       carrying every fourth pending round);
//   (3) W <- F W - Bm X_w,  F = A_end,  Bm[r] = a_r rho_{r,end}   (M x d contraction over B).
// The dependent rounds (2) occupy one wavefront; so that the matrix cores do not wait for them,
// (2) of window k runs beside the sweep that applies (3) of window k - 1.  Its inner products
// cannot then be taken with w_k itself (not formed yet); the sweep before took Q' = W_{k-1} X_k^T,
// and with W_k = F W_{k-1} - Bm X_{k-1},
//     Q0_k = F Q' - Bm (X_{k-1} X_k^T),
// a 16 x 64 x 64 contraction with the cross Gram matrix of the two windows (pre-pass), four
// matrix instructions deep.  One sweep over the coordinates per window, block by block:
// (3) of window k - 1, then that block's share of W_k X_{k+1}^T, so the iterates are touched once
// per window.  ||w||^2 is carried through the windows by the scalar identity above (float64) and
// re-anchored one window late on the exact sum of squares that the sweep takes of the new iterates.
//
// The iterates live in HBM between windows: the sweep loads each 16 x 16 block, updates it, takes
// its share of the next window's inner products and writes it back, 8 bytes per coordinate,
// learner and window, all in full 64-byte segments.  A workgroup works two tiles, so that every
// round row a wavefront loads (from L2: all tiles read the same rows) serves 32 learners; a
// compute unit draws only about 21 bytes per clock from L2, which is what bounds the sweep.
// Variants (OCO_OPT_WINDOW_RESIDENT): the iterates of one tile held in the registers of the
// workgroup for a whole launch (d <= 4096: eight wavefronts, each with every eighth block, in
// the layout the matrix instruction writes: a lane holds 4 coordinates of one learner); those of
// two tiles (d <= 1024; the default for 512 <= d <= 1024: a window's time is then the dependent
// rounds plus the sweep of the wavefronts that ran them, and without the iterates' loads and stores
// the sweep is bound by the matrix instructions of each SIMD); and one streamed tile worked by
// sixteen wavefronts.
//
// v_mfma_f32_16x16x4_f32 computes D = A B + C with A 16x4, B 4x16: lane l supplies
// A[l % 16][l / 16] and B[l / 16][l % 16] and holds D[4 (l / 16) + r][l % 16] in register r.
// A block of iterates is kept as the transposed 16 coordinates x 16 learners D tile, so that
// register r of it is at once the B operand of (1) for the depth indices k <-> coordinate 4 k + r
// (the order of the terms of an inner product is free; the round rows are laid out to match).
//
// The round rows as operands.  In (1) a lane holds (round l % 16, four coordinates): read from
// the stream, neighbouring lanes would sit in different rows, 16 bytes each.  A pre-pass
// therefore re-tiles the stream once per launch: per window and block of 16 coordinates, 4 KB in
// the order the lanes of (1) want them and 4 KB in the order the lanes of (3) want them (lane:
// coordinate l % 16, sixteen rounds), so that every load of the sweep is 16 bytes per lane and
// 1 KB contiguous per instruction, rows past a window's length and coordinates past d already
// zero.  A call is worked in pieces of at most 64 MB of stream so that the two copies stay a
// bounded scratch (and, with the piece itself, inside the last-level cache for every tile).
//
// Windows end at the multiples of 64 of the horizon; a call that starts or ends elsewhere has
// shorter first / last windows.
#include "oco_internal.h"
#include "../../include/oco.h"

#include <algorithm>
#include <cstdio>
#include <type_traits>
#include <utility>

namespace oco {
namespace {

constexpr int kB = 64;            // rounds per window
constexpr int kM = 16;            // learners per tile
constexpr int kNW8 = 8;           // wavefronts per workgroup: iterates in registers (two per SIMD, 256 registers each)
constexpr int kNW16 = 16;         // ... iterates streamed from HBM (four per SIMD: a wavefront's loads hide behind the others' work)
constexpr int kGStride = 18;      // doubles per (round, quad lane) row of the masked Gram table (16 + padding)
constexpr int64_t kPieceBytes = 64ll << 20;   // stream per launch (each tiled copy is as large)
constexpr int kTileFloats = kB * 16;          // one window x one block of 16 coordinates
// A little scratch that lets the streamed sweep load and store without branches (a load or store
// that may or may not have been issued makes every later wait a wait for everything): lanes
// without a learner or past d read kMiscZeros zero floats and write to a sink of their own.
constexpr int kMiscZeros = 16, kMiscFloats = kMiscZeros + 1024 * 4;

typedef float f4 __attribute__((ext_vector_type(4)));

// (A build with -DOCO_WIN_PROF keeps wall-clock sums of the phases of workgroup 0's window loop in g_win_prof,
// read back through oco_debug_win_prof: how the figures per phase in the comments below were taken.)
#ifdef OCO_WIN_PROF
__device__ unsigned long long g_win_prof[8];
#ifndef OCO_WIN_PROF_TID
#define OCO_WIN_PROF_TID 0
#endif
#define PROF_T(i) do { if (threadIdx.x == OCO_WIN_PROF_TID) { const unsigned long long now_ = wall_clock64(); prof_[i] += now_ - last_; last_ = now_; } } while (0)
#else
#define PROF_T(i) do { } while (0)
#endif

struct WinPlanD {
    int64_t t0;      // absolute round of the call's first round
    int n;           // rounds in the call
    __host__ __device__ int first_len() const { const int f = (int)(kB - t0 % kB); return f < n ? f : n; }
    __host__ __device__ int count() const { const int f = first_len(); return 1 + (n - f + kB - 1) / kB; }
    __host__ __device__ int start(int w) const { return w == 0 ? 0 : first_len() + (w - 1) * kB; }
    __host__ __device__ int len(int w) const { const int s = start(w); const int l = w == 0 ? first_len() : kB; return l < n - s ? l : n - s; }
};

template <int LOSS> __device__ __forceinline__ float slope(float z, float y)
{
    if (LOSS == 0) return 1.0f;
    if (LOSS == 1) return 2.0f * (z - y);
    return -y * __builtin_amdgcn_rcpf(1.0f + __expf(y * z));
}

// ---- pre-pass 1: the round rows of the windows w0 .. w0 + gridDim.y - 1, re-tiled ----------------
// One wavefront per (window, block of 16 coordinates).  xq[((w - w0) nblk + blk) 1024 + (rb 64 + l) 4 + r]
// = x[round 16 rb + l % 16][coordinate 16 blk + 4 (l / 16) + r], xu[... + (k 64 + l) 4 + r]
// = x[round 4 (4 k + r) + l / 16][coordinate 16 blk + l % 16]; zero past the window or past d.
__global__ void __launch_bounds__(64) dense_tile_kernel(const float *x, int d, WinPlanD plan, int w0, float *xq, float *xu,
                                                        float *misc)
{
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x < kMiscZeros) misc[threadIdx.x] = 0.f;   // see kMiscZeros
    const int blk = blockIdx.x, w = w0 + blockIdx.y;
    const int nblk = gridDim.x;
    const int ws = plan.start(w), wl = plan.len(w);
    const int l = threadIdx.x, lr = l & 15, lk = l >> 4;
    const int64_t tile = ((int64_t)blockIdx.y * nblk + blk) * kTileFloats;
    const float *xw = x + (int64_t)ws * d + blk * 16;
    {
        const int c = blk * 16 + 4 * lk;
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) {
            const int t = rb * 16 + lr;
            f4 v = f4{0.f, 0.f, 0.f, 0.f};
            if (c < d && t < wl) v = *reinterpret_cast<const f4 *>(xw + (int64_t)t * d + 4 * lk);
            *reinterpret_cast<f4 *>(xq + tile + (rb * 64 + l) * 4) = v;
        }
    }
    {
        const int c = blk * 16 + lr;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            f4 v;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int t = 4 * (4 * k + r) + lk;
                v[r] = (c < d && t < wl) ? xw[(int64_t)t * d + lr] : 0.f;
            }
            *reinterpret_cast<f4 *>(xu + tile + (k * 64 + l) * 4) = v;
        }
    }
}

// ---- pre-pass 2: G = X_w X_w^T of the same windows, from the tiled rows, and the cross Gram
// matrix Gx[r][t] = <x_r of window w - 1, x_t of window w> for every window but the launch's first.
// One workgroup of eight wavefronts per window; wavefronts 0..3 compute rows 16 v .. 16 v + 15 of G
// (four 16 x 16 blocks), wavefronts 4..7 the same rows of Gx, depth block by block.  Fixed
// summation order.  Gx is written in the order the round kernel's matrix instructions want it:
// gxt[((t / 16) 4 + r / 16) 256 + (t % 16 + 16 (r % 4)) 4 + (r / 4) % 4].
__global__ void __launch_bounds__(512) dense_gram_kernel(const float *xq, int nblk, float *gram, float *gxt)
{
    const int lane = threadIdx.x & 63, wave8 = threadIdx.x >> 6;
    const int wave = wave8 & 3;
    const bool cross = wave8 >= 4;
    if (cross && blockIdx.x == 0) return;
    const int lr = lane & 15, lk = lane >> 4;
    f4 acc[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[b] = f4{0.f, 0.f, 0.f, 0.f};
    const float *xw = xq + (int64_t)blockIdx.x * nblk * kTileFloats + lane * 4;          // this window
    const float *xa = cross ? xw - (int64_t)nblk * kTileFloats : xw;                     // rows: the window before, or this one
    for (int blk = 0; blk < nblk; ++blk) {
        f4 bv[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) bv[b] = *reinterpret_cast<const f4 *>(xw + (int64_t)blk * kTileFloats + b * 256);
        const f4 av = *reinterpret_cast<const f4 *>(xa + (int64_t)blk * kTileFloats + wave * 256);
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc[b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[r], bv[b][r], acc[b], 0, 0, 0);
    }
    // acc[b][r]: row 16 wave + 4 lk + r, column 16 b + lr
    if (!cross) {
        float *g = gram + (int64_t)blockIdx.x * kB * kB;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) g[(wave * 16 + 4 * lk + r) * kB + b * 16 + lr] = acc[b][r];
    } else {
        float *g = gxt + (int64_t)blockIdx.x * kB * kB;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
            for (int r = 0; r < 4; ++r) g[(b * 4 + wave) * 256 + (lr + 16 * r) * 4 + lk] = acc[b][r];
    }
}

// LDS of the window kernel (dynamic), in bytes from the base.  What the dependent rounds of window
// k write for the sweep (predictions, -Bm, F) and the labels staged for them have two buffers,
// window k in buffer k % 2: the sweep of window k - 1 and the staging for window k + 1 run beside
// them.  The Gram table (float64, its diagonal in the rows' padding) has one: it is written
// between the two barriers that precede the rounds, from registers loaded before the first.
// MT: tiles of 16 learners per workgroup (per-tile arrays come MT times; the Gram table and the
// shares' buffer are common).
template <int NW, int MT> struct LdsT {
    // float64 where the LDS has room (one tile, eight wavefronts), else float32
    static constexpr bool wide = NW == kNW8 && MT == 1;
    using G = double;                                              // Gram table
    using S = std::conditional_t<wide, double, float>;             // inner products handed to the rounds, f_t
    static constexpr bool has_corr = true;                         // the rounds start from pmul q0 + corr
    static constexpr int gd_bytes = kB * 4 * kGStride * (int)sizeof(G);   // G [64][4][kGStride]: G[t][t2], zero for t2 <= t;
                                                                   //   [t][0][16] holds G[t][t]
    static constexpr int tile_f = kB * kM * 4;                     // float [64][16]
    static constexpr int tile_s = kB * kM * (int)sizeof(S);        // S [64][16]
    static constexpr int yb_bytes = MT * tile_f;                   // labels
    static constexpr int zb_bytes = MT * tile_f;                   // predictions
    static constexpr int bm_bytes = MT * tile_f;                   // -Bm
    static constexpr int fv_bytes = MT * kM * 4;                   // float [16]: F
    static constexpr int gd = 0;
    static constexpr int yb = gd + gd_bytes;
    static constexpr int zb = yb + 2 * yb_bytes;
    static constexpr int bm = zb + 2 * zb_bytes;
    static constexpr int fv = bm + 2 * bm_bytes;
    static constexpr int q0 = fv + 2 * fv_bytes;                   // S [MT][64][16]: W' X_k^T
    static constexpr int fl = q0 + MT * tile_s;                    // S [MT][64][16]: f_t
    static constexpr int part = fl + MT * tile_s;                  // float [NW][64][16]: per-wavefront shares of W X^T (one tile at a time)
    static constexpr int st = part + NW * tile_f;                  // float [MT][64][16]: a_t
    static constexpr int corr = st + MT * tile_f;                  // float [MT][64][16]: -Bm (X_{k-1} X_k^T)
    static constexpr int n2 = corr + MT * tile_f;                  // float [MT][NW][4][16]: shares of ||w||^2
    static constexpr int hg = n2 + MT * NW * 4 * kM * 4;           // float [2][64]: <x_{t-1}, x_t> of the window's rounds (optimistic update)
    static constexpr int hg_bytes = kB * 4;
    static constexpr int total = hg + 2 * hg_bytes;
};
static_assert(LdsT<kNW8, 1>::total <= 160 * 1024 && LdsT<kNW16, 1>::total <= 160 * 1024 && LdsT<kNW8, 2>::total <= 160 * 1024,
              "LDS of a gfx950 compute unit");

// every lane of a quad gets the value of the quad's lane SEL
template <int SEL> __device__ __forceinline__ double quad_bcast(double v)
{
    constexpr int ctrl = SEL * 0x55;                             // quad_perm [SEL, SEL, SEL, SEL]
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), ctrl, 0xF, 0xF, false);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), ctrl, 0xF, 0xF, false);
    return __hiloint2double(hi, lo);
}

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose index is a
// compile-time constant in every iteration (register arrays indexed by it stay in registers)
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F> __device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// The 64 dependent rounds of window k for the tile's 16 learners: wavefront 0, lane = 4 learner
// + quad lane s; quad lane s carries the pending predictions of the rounds t2 = 4 j + s.
// In: q0 = W' X_k^T with W' the iterates before the step of window k - 1 (or the stored ones, for the
// launch's first window), pmul and corr such that pmul q0 + corr = W_k X_k^T; labels, G; n2 = ||w_k||^2.
// Out (LDS buffer k % 2): predictions, -Bm, F = fscale f_0 ... f_63; returns F; n2 becomes ||w_{k+1}||^2
// by the scalar identity, *projected whether any round of the window projected this learner.
// Straight-line code: a window shorter than 64 rounds (first / last window of a call) runs its
// missing rounds as rounds without a step (a = 0, so f = 1 and no pending prediction moves; their
// rows of G are zero).
// The scalars the optimistic update (Eq. (3)) carries from round to round: the hint is ha x_{t-1},
// hp = <w^_t, x_{t-1}>, x2p = ||x_{t-1}||^2 (the vector the sweeps move is then the intermediate model w^).
struct Hint { float ha, hp, x2p; };

template <int LOSS, class Lds, bool OPT = false>
__device__ __forceinline__ double chain_window(char *lds, int buf, int m, int lane, int wl, float eta, double D, double pmul,
                                               double fscale, double &n2, bool &projected, Hint *hint = nullptr)
{
    using GT = typename Lds::G;
    using ST = typename Lds::S;
    const int lc = lane >> 2, s = lane & 3;
    const GT *gd = reinterpret_cast<const GT *>(lds + Lds::gd) + s * kGStride;
    const GT *x2d = reinterpret_cast<const GT *>(lds + Lds::gd) + 16;
    const ST *q0d = reinterpret_cast<const ST *>(lds + Lds::q0 + m * Lds::tile_s) + s * kM + lc;
    const float *cr = reinterpret_cast<const float *>(lds + Lds::corr + m * Lds::tile_f) + s * kM + lc;
    ST *fl = reinterpret_cast<ST *>(lds + Lds::fl + m * Lds::tile_s) + lc;
    const float *yb = reinterpret_cast<const float *>(lds + Lds::yb + buf * Lds::yb_bytes + m * Lds::tile_f) + lc;
    float *zb = reinterpret_cast<float *>(lds + Lds::zb + buf * Lds::zb_bytes + m * Lds::tile_f) + lc;
    float *stl = reinterpret_cast<float *>(lds + Lds::st + m * Lds::tile_f) + lc;
    const float Df = (float)D, D2f = Df * Df;
    const float eta2 = 2.f * eta;
    bool anyp = false;

    double p[16];
#pragma unroll
    for (int j = 0; j < 16; ++j)
        p[j] = Lds::has_corr ? fma(pmul, (double)q0d[4 * j * kM], (double)cr[4 * j * kM]) : pmul * (double)q0d[4 * j * kM];

    // A round has a short dependent part (prediction -> slope -> step -> norm -> projection factor
    // -> next prediction) and a wide independent one (its update of the pending predictions).  The
    // dependent part runs in float32: the next prediction is taken from the float64 pending value
    // by one float32 step, f (p - a G), as exact as a float32 inner product of that size; the
    // squared norm is carried in float32 within the window like the register kernel carries it
    // between its exact measurements (the caller re-anchors it every window).  The pending
    // predictions themselves stay float64 (their recurrence is 64 rounds long); round t - 1's
    // update of them shares a scheduling region with the dependent part of round t and fills its
    // latencies.
    double gprev[16];                 // round t - 1's row of G (elements j >= (t - 1) / 4)
    double aprev = 0.0, fprev = 1.0;
    float n2f = (float)n2;
    float znext = (float)p[0];        // this lane's candidate for the next prediction (round 0: lane 0's is the one)
    // label and ||x||^2 of a round are read from LDS one round ahead: they are the first things the
    // dependent part needs, and nothing else would cover the latency of the read
    float ynext = yb[0], x2next = (float)x2d[0];
    const float *hg = reinterpret_cast<const float *>(lds + Lds::hg + buf * Lds::hg_bytes);
    float gnext = OPT ? hg[0] : 0.f;
    float ha = 0.f, hp = 0.f, x2p = 0.f;
    if (OPT) { ha = hint->ha; hp = hint->hp; x2p = hint->x2p; }
    static_for<kB>([&](auto tc) __attribute__((always_inline)) {
        constexpr int t = decltype(tc)::value;
        constexpr int j0 = t >> 2;                                   // pending elements of this lane: j >= j0
        constexpr int jn = (t + 1) >> 2;                             // holds the prediction of round t + 1
        // this round's row of G first: it does not depend on the scalars below
        double gr[16 - j0];
#pragma unroll
        for (int j = j0; j < 16; ++j) gr[j - j0] = gd[t * 4 * kGStride + j];
        const float yt = ynext, x2t = x2next, g01t = gnext;
        if constexpr (t + 1 < kB) {
            ynext = yb[(t + 1) * kM];
            x2next = (float)x2d[(t + 1) * 4 * kGStride];
            if (OPT) gnext = hg[t + 1];
        }
        if constexpr (t > 0) {
            constexpr int jp0 = (t - 1) >> 2;
#pragma unroll
            for (int j = jp0; j < 16; ++j) p[j] = fprev * fma(-aprev, gprev[j], p[j]);
        }
        const float z32 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(znext), (t & 3) * 0x55, 0xF, 0xF, false));   // <w_t, x_t>
        // the prediction that is played and scored: plain, z32; optimistic, that of w_t = s (w^_t - ha x_{t-1})
        // with s from ||w^_t - ha x_{t-1}||^2, all from scalars (z32 is then <w^_t, x_t>)
        float zp = z32;
        if (OPT) {
            const float mf = fmaf(ha * ha, x2p, fmaf(-2.f * ha, hp, n2f));
            const float sp = mf > D2f ? Df * __builtin_amdgcn_rsqf(mf) : 1.f;
            zp = sp * fmaf(-ha, g01t, z32);
        }
        // a_t = eta c_t; for the squared loss eta * 2 (z - y) = (2 eta) (z - y) exactly
        float a32 = LOSS == 1 ? eta2 * (zp - yt) : eta * slope<LOSS>(zp, yt);
        a32 = t < wl ? a32 : 0.f;
        // ||w_t - a_t x_t||^2 and the projection factor
        const float m2 = fmaxf(fmaf(a32, fmaf(a32, x2t, -2.f * z32), n2f), 0.f);
        const bool pj = m2 > D2f;
        const float f32v = pj ? Df * __builtin_amdgcn_rsqf(m2) : 1.f;
        n2f = pj ? D2f : m2;
        anyp = anyp || pj;
        zb[t * kM] = zp;                                             // (the quad's four lanes write the same value)
        stl[t * kM] = a32;
        fl[t * kM] = (ST)f32v;
        if (OPT) {                                                   // next round's hint and <w^_{t+1}, x_t>
            const bool live = t < wl;                                // (selects, not a branch: the rounds stay straight-line code)
            hp = live ? f32v * fmaf(-a32, x2t, z32) : hp;
            ha = live ? a32 : ha;
            x2p = live ? x2t : x2p;
        }
        // (p[jn] has the updates of the rounds before this one: the loop above ran)
        if constexpr (jn < 16) znext = f32v * fmaf(-a32, (float)gr[jn - j0], (float)p[jn]);
#pragma unroll
        for (int j = j0; j < 16; ++j) gprev[j] = gr[j - j0];
        aprev = (double)a32;
        fprev = (double)f32v;
        __builtin_amdgcn_sched_barrier(0);                           // at most two rounds overlap: registers
    });
    n2 = (double)n2f;
    if (OPT) { hint->ha = ha; hint->hp = hp; hint->x2p = x2p; }

    // Bm[r] = a_r f_r f_{r+1} ... f_63 and F = fscale f_0 ... f_63: quad lane s takes the rounds
    // 16 s .. 16 s + 15 backwards, then the quad's products are combined
    float *bm = reinterpret_cast<float *>(lds + Lds::bm + buf * Lds::bm_bytes + m * Lds::tile_f) + lc;
    float *fv = reinterpret_cast<float *>(lds + Lds::fv + buf * Lds::fv_bytes) + m * kM;
    double loc[16];
    double acc = 1.0;
#pragma unroll
    for (int k = 15; k >= 0; --k) {
        acc *= (double)fl[(16 * s + k) * kM];
        loc[k] = acc;
    }
    const double P0 = quad_bcast<0>(acc), P1 = quad_bcast<1>(acc), P2 = quad_bcast<2>(acc), P3 = quad_bcast<3>(acc);
    const double tail = s == 3 ? 1.0 : s == 2 ? P3 : s == 1 ? P2 * P3 : P1 * (P2 * P3);
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        const int r = 16 * s + k;
        bm[r * kM] = -(float)((double)stl[r * kM] * (loc[k] * tail));
    }
    const double F = fscale * (P0 * (P1 * (P2 * P3)));
    if (s == 0) fv[lc] = (float)F;
    projected = anyp;
    return F;
}

// What a thread is in the sweep, derived from its index.  The window loop re-derives it every
// iteration from an index the compiler cannot see through, so that none of it (nor the many
// addresses that follow from it) is kept alive across the dependent rounds.
template <int MT> struct Geo {
    int tid, lane, wave, lr, lk;
    bool q_ok[MT];             // this lane's learner of tile m exists
    float *vrow[MT];           // its row of the iterates, at this lane's 4 coordinates of a block
};
template <int MT> __device__ __forceinline__ Geo<MT> make_geo(int tid, const DenseArgs &a)
{
    Geo<MT> g;
    g.tid = tid;
    g.lane = tid & 63;
    g.wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    g.lr = g.lane & 15;
    g.lk = g.lane >> 4;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int q = ((int)blockIdx.x * MT + m) * kM + g.lr;
        g.q_ok[m] = q < a.R * a.K;
        g.vrow[m] = a.V + (int64_t)(g.q_ok[m] ? q : 0) * a.d + 4 * g.lk;
    }
    return g;
}

// The windows w0 .. w0 + nw - 1 of the call's plan; xq / xu / gram / gxt hold those windows only.
// RES: the iterates stay in registers for the whole launch (one tile, d <= 16 * NW * NB); otherwise
// every block is loaded and stored in the sweep.  NW: wavefronts per workgroup.  MT: tiles of 16
// learners per workgroup -- with two, a wavefront uses every round row it loads for both (a compute
// unit draws only about 21 bytes per clock from L2, and the sweep of one tile needs 8 KB of rows per
// 32 matrix instructions); wavefront m runs the dependent rounds of tile m.
//
// Iteration k = 0 .. nw of the main loop:
//   all        the shares of W' X_k^T -> q0, tile by tile; four wavefronts per tile: corr = -Bm_{k-1} Gx_k (k >= 1)
//   wavefronts < MT    the dependent rounds of window k (k < nw), then their part of the sweep
//   the others     predictions of window k - 1 to Z, staging for window k + 1, the sweep
//   sweep (k >= 1) W_k = F_{k-1} W_{k-1} - Bm_{k-1} X_{k-1} block by block, its squared norm, and the
//                  shares of W_k X_{k+1}^T (k + 1 < nw)
template <int LOSS, int NB, bool RES, int NW, int MT, bool OPT = false>
__global__ void __launch_bounds__(NW *kWave) dense_window_kernel(const DenseArgs a, const float *gram, const float *gxt,
                                                                  const float *xq, const float *xu, float *misc,
                                                                  WinPlanD plan, int w0, int nw)
{
    static_assert(!RES || MT == 1 || (MT == 2 && NW == 8 && NB == 9), "iterates in registers: one tile, or two on eight wavefronts");
    using Lds = LdsT<NW, MT>;
    using GT = typename Lds::G;
    using ST = typename Lds::S;
    // -Bm in registers for the whole sweep, or (where registers are short) re-read from LDS per block
    constexpr bool BMR = RES && NB <= 8 && MT == 1;
    extern __shared__ __align__(16) char lds[];
    const int d = a.d, K = a.K;
    const int nq = a.R * K;
    const int nblk = (d + 15) / 16;                             // blocks of 16 coordinates
    const int q_base = (int)blockIdx.x * MT * kM;               // first learner of the workgroup

    // Which blocks of 16 coordinates a wavefront takes.  In registers: wave, wave + NW, ...  Streamed
    // with sixteen wavefronts: wavefront 0 also runs the dependent rounds, so it takes half a share:
    // of every 31 consecutive blocks, wavefronts 1 .. 15 take two each and wavefront 0 the last one.
    // (A fixed assignment: every sum keeps its order from run to run.)
    auto nth_block = [&](int wave, int i) __attribute__((always_inline)) {
        if (NW == kNW16 && !RES) {
            if (wave == 0) return 31 * i + 30;
            return 31 * (i >> 1) + (wave - 1) + ((i & 1) ? 15 : 0);
        }
        if (MT == 2) {
            // two tiles, eight wavefronts: wavefronts 0 and 1 run the dependent rounds first and take two
            // blocks of every 22, the other six three each
            if (wave < 2) return 22 * (i >> 1) + 6 + wave + 8 * (i & 1);
            return 22 * (i / 3) + (wave - 2) + 8 * (i % 3);
        }
        return wave + NW * i;
    };
    // Which wavefront runs the dependent rounds of which tile (-1: of none), and the number of a wavefront
    // among those that run none.  Two tiles in registers: wavefronts 0 and 4, which share a SIMD (a workgroup's
    // wavefronts are dealt to the four SIMDs in turn), so that the rounds do not share theirs with a wavefront
    // of matrix instructions (beside one they take 16 us per window instead of 10) and the other three SIMDs
    // have two sweeping wavefronts each.
    constexpr bool PAIR = RES && MT == 2;
    auto rounds_tile = [&](int wave) __attribute__((always_inline)) {
        if (PAIR) return (wave & 3) == 0 ? wave >> 2 : -1;
        return wave < MT ? wave : -1;
    };
    auto other_index = [&](int wave) __attribute__((always_inline)) {
        if (PAIR) return wave < 4 ? wave - 1 : wave - 2;
        return wave - MT;
    };
    // Iterates in registers: the b-th block a wavefront keeps.  One tile: wave, wave + NW, ...  Two tiles
    // (eight wavefronts, NB = 9, at most 64 blocks): the six wavefronts without dependent rounds keep blocks
    // 0 .. 53, nine each; the two with them sweep only when their rounds are done and keep blocks 54 .. 63:
    // wavefront 0, whose rounds the SIMD works first, seven of them, wavefront 4 three.
    auto kept_block = [&](int wave, int b) __attribute__((always_inline)) {
        if (PAIR) {
            if ((wave & 3) != 0) return other_index(wave) + 6 * b;
            return wave == 0 ? (b < 7 ? 54 + b : (1 << 20)) : (b < 3 ? 61 + b : (1 << 20));
        }
        return wave + NW * b;
    };
    // a tile's iterates: 16 coordinates x 16 learners per block, transposed
    auto ld_block = [&](const Geo<MT> &g, int m, int blk) __attribute__((always_inline)) {
        f4 v = f4{0.f, 0.f, 0.f, 0.f};
        if (g.q_ok[m] && blk * 16 + 4 * g.lk < d) v = *reinterpret_cast<const f4 *>(g.vrow[m] + blk * 16);
        return v;
    };
    auto st_block = [&](const Geo<MT> &g, int m, int blk, const f4 &v) __attribute__((always_inline)) {
        if (g.q_ok[m] && blk * 16 + 4 * g.lk < d) *reinterpret_cast<f4 *>(g.vrow[m] + blk * 16) = v;
    };
    // the same without a branch (streamed sweep): every lane loads and stores, the lanes without a
    // learner or past d from / to the scratch words
    auto ld_block_nb = [&](const Geo<MT> &g, int m, int blk) __attribute__((always_inline)) {
        const bool ok = g.q_ok[m] && blk * 16 + 4 * g.lk < d;
        const float *src = ok ? g.vrow[m] + blk * 16 : misc;
        return *reinterpret_cast<const f4 *>(src);
    };
    auto st_block_nb = [&](const Geo<MT> &g, int m, int blk, const f4 &v) __attribute__((always_inline)) {
        const bool ok = g.q_ok[m] && blk * 16 + 4 * g.lk < d;
        float *dst = ok ? g.vrow[m] + blk * 16 : misc + kMiscZeros + g.tid * 4;
        *reinterpret_cast<f4 *>(dst) = v;
    };
    // the tiled round rows of window wi (relative to w0), block blk: four 16-byte loads per lane each
    auto ldq = [&](const Geo<MT> &g, int wi, int blk, f4 (&o)[4]) __attribute__((always_inline)) {
        const float *t = xq + ((int64_t)wi * nblk + blk) * kTileFloats + g.lane * 4;
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) o[rb] = *reinterpret_cast<const f4 *>(t + rb * 256);
    };
    auto ldu = [&](const Geo<MT> &g, int wi, int blk, f4 (&o)[4]) __attribute__((always_inline)) {
        const float *t = xu + ((int64_t)wi * nblk + blk) * kTileFloats + g.lane * 4;
#pragma unroll
        for (int k = 0; k < 4; ++k) o[k] = *reinterpret_cast<const f4 *>(t + k * 256);
    };
    // The Gram matrix of window wi on its way to LDS: every thread carries kGPer consecutive entries
    // of a row in registers (loaded before a barrier, stored after it), masked to t2 > t, the
    // diagonal in the rows' padding.
    constexpr int kGPer = kB * kB / (NW * kWave);               // 8 or 4
    auto load_gram = [&](int tid, int wi, f4 (&gv)[kGPer / 4]) __attribute__((always_inline)) {
        const float *gsrc = gram + (int64_t)wi * kB * kB + tid * kGPer;
#pragma unroll
        for (int i = 0; i < kGPer / 4; ++i) gv[i] = *reinterpret_cast<const f4 *>(gsrc + 4 * i);
    };
    auto store_gram = [&](int tid, const f4 (&gv)[kGPer / 4]) __attribute__((always_inline)) {
        GT *gd = reinterpret_cast<GT *>(lds + Lds::gd);
        const int t = (tid * kGPer) >> 6, t2b = (tid * kGPer) & 63;
#pragma unroll
        for (int i = 0; i < kGPer; ++i) {
            const int t2 = t2b + i;
            const float v = gv[i >> 2][i & 3];
            gd[(t * 4 + (i & 3)) * kGStride + (t2 >> 2)] = t2 > t ? (GT)v : (GT)0;   // (t2b is a multiple of 4: t2 & 3 == i & 3)
            if (t2 == t) gd[t * 4 * kGStride + 16] = (GT)v;
        }
    };
    // LDS inputs of the dependent rounds of window wi: the labels.  `nthr` threads numbered tid share the work.
    auto stage_chain_inputs = [&](int tid, int nthr, int wi) __attribute__((always_inline)) {
        const int w = w0 + wi, buf = wi & 1;
        const int ws = plan.start(w), wl = plan.len(w);
        float *yb = reinterpret_cast<float *>(lds + Lds::yb + buf * Lds::yb_bytes);
        for (int e = tid; e < MT * kB * kM; e += nthr) {
            const int l = e >> 6, t = e & 63;                   // a learner's 64 labels are contiguous
            const int q = q_base + l;
            float yv = 0.f;
            if (a.y && q < nq && t < wl) yv = a.y[(int64_t)(q / K) * a.y_run_stride + ws + t];
            yb[((l >> 4) * kB + t) * kM + (l & 15)] = yv;
        }
        if (OPT) {
            float *hg = reinterpret_cast<float *>(lds + Lds::hg + buf * Lds::hg_bytes);
            for (int t = tid; t < kB; t += nthr) hg[t] = t < wl ? a.g01[ws + t] : 0.f;
        }
    };
    // shares of this wavefront of one tile's W X^T for one window -> LDS
    auto put_part = [&](const Geo<MT> &g, const f4 (&acc)[4]) __attribute__((always_inline)) {
        float *part = reinterpret_cast<float *>(lds + Lds::part);
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
            for (int r = 0; r < 4; ++r) part[(g.wave * kB + rb * 16 + 4 * g.lk + r) * kM + g.lr] = acc[rb][r];
    };
    // tile m's W' X_k^T = sum of the wavefronts' shares, fixed order, summed in float64
    auto sum_parts = [&](int tid, int m) __attribute__((always_inline)) {
        const float *part = reinterpret_cast<const float *>(lds + Lds::part);
        ST *q0d = reinterpret_cast<ST *>(lds + Lds::q0 + m * Lds::tile_s);
#pragma unroll
        for (int u = 0; u < kB * kM / (NW * kWave); ++u) {
            const int e = tid + u * NW * kWave;
            double sum = 0.0;
#pragma unroll
            for (int v = 0; v < NW; ++v) sum += (double)part[v * kB * kM + e];
            q0d[e] = (ST)sum;
        }
    };
    // ||w||^2 of tile m's learner lc as the last sweep measured it: 4 NW shares, fixed order
    auto measured_n2 = [&](int m, int lc) __attribute__((always_inline)) {
        const float *n2s = reinterpret_cast<const float *>(lds + Lds::n2) + m * NW * 4 * kM;
        double v = 0.0;
#pragma unroll
        for (int i = 0; i < NW * 4; ++i) v += (double)n2s[i * kM + lc];
        return v;
    };

    // ---- per-learner state of the dependent rounds (wavefront m < MT: lane = 4 learner + quad lane) ----
    float eta = 0.f;
    double pmul = 1.0;          // scale of the iterates q0 was taken with: sigma of the state, then F of the window before
    double n2 = 0.0;            // ||w_k||^2 as the scalar identity carries it
    double n2_begin = 0.0;      // what the previous window's rounds started from
    bool proj_prev = true;      // whether they projected this learner (then n2 was reset to D^2 on the way)
    Hint hint{0.f, 0.f, 0.f};   // optimistic update: carried from round to round, window to window, call to call
    f4 V[RES ? NB : 1][MT];     // iterates in registers: the blocks kept_block() names, of every tile
    f4 accq[MT][4];             // this wavefront's shares of W_k X_{k+1}^T; tile 0's go to LDS at once, the others wait their turn
    {
        const Geo<MT> g = make_geo<MT>((int)threadIdx.x, a);
        const int q_ch = q_base + rounds_tile(g.wave) * kM + (g.lane >> 2);
        if (rounds_tile(g.wave) >= 0 && q_ch < nq) {
            eta = a.eta[q_ch % K];
            pmul = (double)a.sigma[q_ch];
            n2 = a.n2[q_ch] * pmul * pmul;                      // ||w||^2 of the iterate itself
            if (OPT) {
                const int ws0 = plan.start(w0);
                hint.ha = a.ha[q_ch];
                hint.hp = a.hp[q_ch];
                hint.x2p = ws0 == 0 ? a.x2last[0] : a.x2[ws0 - 1];
            }
        }
        if (RES) {
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int m = 0; m < MT; ++m) V[b][m] = ld_block(g, m, kept_block(g.wave, b));
        }
        // ---- prologue: the stored iterates times the rows of the first two windows -----------------
        f4 acc0[MT][4];
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) { acc0[m][rb] = f4{0.f, 0.f, 0.f, 0.f}; accq[m][rb] = f4{0.f, 0.f, 0.f, 0.f}; }
        auto q_of = [&](const f4 (&vb)[MT], int blk) __attribute__((always_inline)) {
            f4 xr[4];
            ldq(g, 0, blk, xr);
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int r = 0; r < 4; ++r)
#pragma unroll
                    for (int rb = 0; rb < 4; ++rb)
                        acc0[m][rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(xr[rb][r], vb[m][r], acc0[m][rb], 0, 0, 0);
            if (nw > 1) {
                ldq(g, 1, blk, xr);
#pragma unroll
                for (int m = 0; m < MT; ++m)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
#pragma unroll
                        for (int rb = 0; rb < 4; ++rb)
                            accq[m][rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(xr[rb][r], vb[m][r], accq[m][rb], 0, 0, 0);
            }
        };
        if constexpr (RES) {
            static_for<NB>([&](auto bc) __attribute__((always_inline)) {
                constexpr int b = decltype(bc)::value;
                const int blk = kept_block(g.wave, b);
                if (blk < nblk) q_of(V[b], blk);
            });
        } else {
            for (int i = 0, blk = nth_block(g.wave, 0); blk < nblk; blk = nth_block(g.wave, ++i)) {
                f4 vb[MT];
#pragma unroll
                for (int m = 0; m < MT; ++m) vb[m] = ld_block(g, m, blk);
                q_of(vb, blk);
            }
        }
        stage_chain_inputs(g.tid, NW * kWave, 0);
        {
            f4 gv[kGPer / 4];
            load_gram(g.tid, 0, gv);
            store_gram(g.tid, gv);
        }
        float *corr = reinterpret_cast<float *>(lds + Lds::corr);
        for (int e = g.tid; e < MT * kB * kM; e += NW * kWave) corr[e] = 0.f;
        // the shares of window 0 are summed here, tile by tile, so that those of window 1 can take their place
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            put_part(g, acc0[m]);
            __syncthreads();
            sum_parts(g.tid, m);
            __syncthreads();
        }
        if (nw > 1) put_part(g, accq[0]);
    }

#ifdef OCO_WIN_PROF
    unsigned long long prof_[8] = {0, 0, 0, 0, 0, 0, 0, 0}, last_ = wall_clock64();
#endif
    for (int k = 0; k <= nw; ++k) {
        int tid_w = (int)threadIdx.x;
        asm volatile("" : "+v"(tid_w));                          // see Geo
        const bool rounds = k < nw;                              // this iteration has dependent rounds (window k)
        const bool sweep = k >= 1;                               // ... and a sweep (window k - 1)
        const bool more = k + 1 < nw;                            // the sweep also takes W_k X_{k+1}^T
        // the cross Gram matrix of windows k - 1 and k as matrix operand, on its way across the barrier
        f4 gx[4];
        const int wave_w = __builtin_amdgcn_readfirstlane(tid_w >> 6);
        const bool corr_wave = rounds && sweep && wave_w < 4 * MT;   // four wavefronts per tile
        if (corr_wave) {
            const float *t = gxt + (int64_t)k * kB * kB + (wave_w & 3) * 1024 + (tid_w & 63) * 4;
#pragma unroll
            for (int j = 0; j < 4; ++j) gx[j] = *reinterpret_cast<const f4 *>(t + j * 256);
        }
        f4 gpre[kGPer / 4];
        const bool gram_now = rounds && k >= 1;                  // (window 0's table: prologue)
        if (gram_now) load_gram(tid_w, k, gpre);
        __syncthreads();                                         // (A) shares of W' X_k^T, -Bm_{k-1}, staged inputs in LDS
        PROF_T(0);
        if (gram_now) store_gram(tid_w, gpre);                   // (the rounds of window k - 1 are long done with theirs)
        if (rounds && k >= 1) {                                  // (window 0: summed in the prologue)
            sum_parts(tid_w, 0);
            if (MT > 1) {
                const Geo<MT> g1 = make_geo<MT>(tid_w, a);
#pragma unroll
                for (int m = 1; m < MT; ++m) {
                    __syncthreads();
                    put_part(g1, accq[m]);
                    __syncthreads();
                    sum_parts(tid_w, m);
                }
            }
        }
        if (corr_wave) {
            // corr[t][learner] = -sum_r Bm_{k-1}[r][learner] Gx[r][t], rows t = 16 (wave % 4) .. + 15, tile wave / 4
            const int m = wave_w >> 2, rbw = wave_w & 3;
            const float *bmp = reinterpret_cast<const float *>(lds + Lds::bm + ((k - 1) & 1) * Lds::bm_bytes + m * Lds::tile_f);
            const int lr = tid_w & 15, lk = (tid_w & 63) >> 4;
            f4 c = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int rs = 0; rs < 16; ++rs)
                c = __builtin_amdgcn_mfma_f32_16x16x4f32(gx[rs >> 2][rs & 3], bmp[(rs * 4 + lk) * kM + lr], c, 0, 0, 0);
            float *corr = reinterpret_cast<float *>(lds + Lds::corr + m * Lds::tile_f);
#pragma unroll
            for (int r = 0; r < 4; ++r) corr[(rbw * 16 + 4 * lk + r) * kM + lr] = c[r];
        }
        __syncthreads();                                         // (B)
        PROF_T(1);
        const int tile_w = rounds_tile(wave_w);
        if (tile_w >= 0) {
            if (rounds) {
                const int lane = tid_w & 63;
                if (k >= 2) {
                    // ||w_{k-1}||^2 as the sweep of window k - 2 measured it against what the rounds of window
                    // k - 1 started from: the difference (float32 rounding of the sweeps) went through those
                    // rounds added to every squared norm, and every projection among them scaled it by f^2
                    // (to first order), so F_{k-1}^2 of it is still in the iterate and missing from n2.  The
                    // next projection then removes it from the iterate as well.
                    n2 = fma(measured_n2(tile_w, lane >> 2) - n2_begin, pmul * pmul, n2);
                    n2 = n2 > 0.0 ? n2 : 0.0;
                }
                n2_begin = n2;
                const double fscale = k == 0 ? pmul : 1.0;
                pmul = chain_window<LOSS, Lds, OPT>(lds, k & 1, tile_w, lane, plan.len(w0 + k), eta, (double)a.D, pmul, fscale,
                                                       n2, proj_prev, &hint);
            }
        } else {
            const int tid_o = other_index(wave_w) * kWave + (tid_w & 63), nthr_o = (NW - MT) * kWave;
            // beside the dependent rounds: the next window's labels and Gram table into the other buffer
            if (more) stage_chain_inputs(tid_o, nthr_o, k + 1);
            // ... and the predictions of window k - 1 to Z (a learner's rounds contiguous)
            if (sweep) {
                const int w = w0 + k - 1;
                const int ws = plan.start(w), wl = plan.len(w);
                const float *zb = reinterpret_cast<const float *>(lds + Lds::zb + ((k - 1) & 1) * Lds::zb_bytes);
                for (int e = tid_o; e < MT * kB * kM; e += nthr_o) {
                    const int l = e >> 6, t = e & 63;
                    const int q = q_base + l;
                    if (q < nq && t < wl)
                        a.Z[(int64_t)(q / K) * a.zl.zs_r + (int64_t)(q % K) * a.zl.zs_i + (int64_t)(ws + t) * a.zl.zs_t] =
                            zb[((l >> 4) * kB + t) * kM + (l & 15)];
                }
            }
        }
        PROF_T(2);
        asm volatile("" : "+v"(tid_w));
        const Geo<MT> g = make_geo<MT>(tid_w, a);
        const int lr = g.lr, lk = g.lk;

        // ---- sweep: (3) of window k - 1 and W_k X_{k+1}^T, block by block ------------------------------
        if (sweep) {
            const int wi = k - 1;
            const float *bml = reinterpret_cast<const float *>(lds + Lds::bm + (wi & 1) * Lds::bm_bytes);
            float bmr[MT][BMR ? 16 : 1];
            float F[MT];
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                if (BMR) {
#pragma unroll
                    for (int rs = 0; rs < 16; ++rs) bmr[m][rs] = bml[m * kB * kM + (rs * 4 + lk) * kM + lr];
                }
                F[m] = reinterpret_cast<const float *>(lds + Lds::fv + (wi & 1) * Lds::fv_bytes)[m * kM + lr];
            }
            f4 acc[MT][4];
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) acc[m][rb] = f4{0.f, 0.f, 0.f, 0.f};
            float nn[MT];
#pragma unroll
            for (int m = 0; m < MT; ++m) nn[m] = 0.f;
            struct BlkIn { f4 xu[4]; f4 xq[4]; f4 vb[MT]; };
            const int wq = more ? k + 1 : k;                     // (no window after the last: any rows, unused)
            auto load_in = [&](BlkIn &in, int blk) __attribute__((always_inline)) {
                if constexpr (RES) {
                    if (blk < nblk) {
                        ldu(g, wi, blk, in.xu);
                        if (more) ldq(g, k + 1, blk, in.xq);
                    }
                } else {
                    // no branch around a load: a block past the end reads the last one again
                    const int b = blk < nblk ? blk : nblk - 1;
                    ldu(g, wi, b, in.xu);
                    ldq(g, wq, b, in.xq);
#pragma unroll
                    for (int m = 0; m < MT; ++m) in.vb[m] = ld_block_nb(g, m, b);
                }
            };
            auto compute = [&](BlkIn &in, f4 (&vreg)[MT], int blk) __attribute__((always_inline)) {
                f4 vb[MT], vo[MT];                               // per tile two chains of eight dependent instructions
#pragma unroll
                for (int m = 0; m < MT; ++m) {
                    vb[m] = RES ? vreg[m] : in.vb[m];
                    vo[m] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int r = 0; r < 4; ++r) vb[m][r] *= F[m];
                }
#pragma unroll
                for (int rs = 0; rs < 16; rs += 2)
#pragma unroll
                    for (int m = 0; m < MT; ++m) {
                        const float b0 = BMR ? bmr[m][BMR ? rs : 0] : bml[m * kB * kM + (rs * 4 + lk) * kM + lr];
                        const float b1 = BMR ? bmr[m][BMR ? rs + 1 : 0] : bml[m * kB * kM + ((rs + 1) * 4 + lk) * kM + lr];
                        vb[m] = __builtin_amdgcn_mfma_f32_16x16x4f32(in.xu[rs >> 2][rs & 3], b0, vb[m], 0, 0, 0);
                        vo[m] = __builtin_amdgcn_mfma_f32_16x16x4f32(in.xu[rs >> 2][(rs & 3) + 1], b1, vo[m], 0, 0, 0);
                    }
#pragma unroll
                for (int m = 0; m < MT; ++m) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) vb[m][r] += vo[m][r];
#pragma unroll
                    for (int r = 0; r < 4; ++r) nn[m] = fmaf(vb[m][r], vb[m][r], nn[m]);
                    if (RES) vreg[m] = vb[m]; else st_block_nb(g, m, blk, vb[m]);
                }
                if (more) {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
#pragma unroll
                        for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                            for (int m = 0; m < MT; ++m)
                                acc[m][rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(in.xq[rb][r], vb[m][r], acc[m][rb], 0, 0, 0);
                }
            };
            f4 none[MT];
            if constexpr (RES) {
                // The round rows of the next block are on their way while the matrix instructions of the
                // current block run.
                BlkIn in[2];
                load_in(in[0], kept_block(g.wave, 0));
                static_for<NB>([&](auto bc) __attribute__((always_inline)) {
                    constexpr int b = decltype(bc)::value;
                    const int blk = kept_block(g.wave, b);
                    if (b + 1 < NB) load_in(in[(b + 1) & 1], kept_block(g.wave, b + 1));
                    __builtin_amdgcn_sched_barrier(0);
                    if (blk < nblk) compute(in[b & 1], V[b], blk);
                    __builtin_amdgcn_sched_barrier(0);
                });
            } else if constexpr (NW == kNW16) {
                // One set of input registers: a block's loads are issued when the block before it is
                // done, and the other three wavefronts of the SIMD keep the matrix cores busy meanwhile.
                BlkIn in;
                for (int i = 0, blk = nth_block(g.wave, 0); blk < nblk; blk = nth_block(g.wave, ++i)) {
                    load_in(in, blk);
                    __builtin_amdgcn_sched_barrier(0);
                    compute(in, none, blk);
                    __builtin_amdgcn_sched_barrier(0);
                }
            } else {
                // Two sets of input registers: the next block's loads are in flight during a block's
                // matrix instructions.  No load or store of the loop sits under a branch, so that every
                // wait leaves exactly the younger ones outstanding (the block's two stores and the eleven
                // loads of the next block).
                BlkIn in[2];
                int i = 0;
                load_in(in[0], nth_block(g.wave, 0));
                // (the loop is entered the way it is re-entered, with MT stores younger than the loads:
                // the wait at its head is computed from both and would otherwise drain the stores)
#pragma unroll
                for (int m = 0; m < MT; ++m)
                    *reinterpret_cast<f4 *>(misc + kMiscZeros + m * 2048 + g.tid * 4) = f4{0.f, 0.f, 0.f, 0.f};
                for (; nth_block(g.wave, i + 1) < nblk; i += 2) {
                    load_in(in[1], nth_block(g.wave, i + 1));
                    __builtin_amdgcn_sched_barrier(0);
                    compute(in[0], none, nth_block(g.wave, i));
                    __builtin_amdgcn_sched_barrier(0);
                    load_in(in[0], nth_block(g.wave, i + 2));
                    __builtin_amdgcn_sched_barrier(0);
                    compute(in[1], none, nth_block(g.wave, i + 1));
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (nth_block(g.wave, i) < nblk) compute(in[0], none, nth_block(g.wave, i));
            }
            PROF_T(4);
#pragma unroll
            for (int m = 0; m < MT; ++m)
                reinterpret_cast<float *>(lds + Lds::n2)[m * NW * 4 * kM + (g.wave * 4 + lk) * kM + lr] = nn[m];
            if (more) {
#pragma unroll
                for (int m = 0; m < MT; ++m)
#pragma unroll
                    for (int rb = 0; rb < 4; ++rb) accq[m][rb] = acc[m][rb];
                put_part(g, accq[0]);
            }
        }
        PROF_T(5);
    }
#ifdef OCO_WIN_PROF
    if (threadIdx.x == OCO_WIN_PROF_TID && blockIdx.x == 0)
        for (int i = 0; i < 8; ++i) g_win_prof[i] = prof_[i];
#endif

    // ---- state out: the iterates themselves (scale 1) and their squared norms ---------------------
    {
        const Geo<MT> g = make_geo<MT>((int)threadIdx.x, a);
        if (RES) {
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
                for (int m = 0; m < MT; ++m) st_block(g, m, kept_block(g.wave, b), V[b][m]);
        }
        __syncthreads();
        const int q_ch = q_base + rounds_tile(g.wave) * kM + (g.lane >> 2);
        if (rounds_tile(g.wave) >= 0 && (g.lane & 3) == 0 && q_ch < nq) {
            a.sigma[q_ch] = 1.f;
            a.n2[q_ch] = measured_n2(rounds_tile(g.wave), g.lane >> 2);
            if (OPT) { a.ha[q_ch] = hint.ha; a.hp[q_ch] = hint.hp; }
        }
    }
}

// ---- the same windows with rows and iterates brought to LDS by wavefronts of their own -----------
// Four tiles of 16 learners per workgroup, two working wavefronts per tile (wavefront tau + 4 sigma:
// tile tau, blocks 2 s + sigma), and four wavefronts that only load.  All step through the blocks
// together, one barrier per step.  The loaders bring to a ring of three LDS stages the rows of
// the step's two blocks -- window k's in the lane order of (3), window k + 1's in that of (1) --
// which serve all four tiles (4 KB of L2 traffic per tile and block where a wavefront that loads
// its own rows needs 8 KB), and the eight blocks of iterates of the step; their registers are the
// prefetch buffer (the loads of four steps are on their way).  The working wavefronts read the
// operands of step s + 1 from LDS while the matrix instructions of step s run, and store the
// new block; they never wait for a memory instruction.  (On this hardware one counter per
// wavefront covers loads and stores alike and runs in issue order, so a wavefront that stores
// cannot wait for a younger load without also waiting for the acknowledgement of every older
// store, several microseconds here.)
// Windows are not overlapped here: sweep k (step (3) of window k, then W X^T for window k + 1)
// follows the dependent rounds of window k, which wavefront tau runs for tile tau; the inner
// products they start from are exact (no cross-Gram correction) and ||w||^2 is the sum of squares
// the sweep has just taken.  Wavefronts of the workgroup exchange data through LDS only, except
// that the loaders read iterates the others stored one sweep earlier (they wait for those stores
// once per window, after the dependent rounds); the barriers are therefore bare s_barrier
// instructions behind a wait for the LDS operations of the wavefront (__syncthreads() would also
// wait for every store's acknowledgement).
// Measured on c4 (one workgroup per compute unit, 128 steps per window): 1.07 us per step with the
// loads switched off against 0.85 us of matrix instructions, 1.35 us with them, whether the
// loads go through registers or straight to LDS and whatever their distance; the dependent rounds
// (not overlapped) and the hand-over between the phases add 35 us per window.
constexpr int kQT = 4, kQS = 2;              // tiles per workgroup, working wavefronts per tile
constexpr int kQW = kQT * kQS;               // working wavefronts; wavefront kQW loads
constexpr int kQStages = 3;
constexpr int kQL = 4, kQSets = 4;           // loading wavefronts; steps of loads each keeps in registers
struct LdsQ {
    using G = double;
    using S = float;
    static constexpr bool has_corr = false;
    static constexpr int gd_bytes = kB * 4 * kGStride * 8;
    static constexpr int tile_f = kB * kM * 4, tile_s = tile_f;
    static constexpr int yb_bytes = kQT * tile_f, zb_bytes = kQT * tile_f, bm_bytes = kQT * tile_f, fv_bytes = kQT * kM * 4;
    static constexpr int rows_bytes = kQS * 2 * 4096;              // per step and block: rows for (3), rows for (1)
    static constexpr int stage_bytes = rows_bytes + kQW * 1024;    // ... and a block of iterates per working wavefront
    static constexpr int gd = 0;
    static constexpr int yb = gd + gd_bytes;
    static constexpr int zb = yb + yb_bytes;
    static constexpr int bm = zb + zb_bytes;
    static constexpr int fv = bm + bm_bytes;
    static constexpr int n2 = fv + fv_bytes;                       // float [kQT][kQS * 4][16]: shares of ||w||^2
    static constexpr int hg = n2 + kQT * kQS * 4 * kM * 4;         // float [64]: <x_{t-1}, x_t> of the window's rounds (optimistic update)
    static constexpr int hg_bytes = kB * 4;
    static constexpr int ring = hg + hg_bytes;
    // between two sweeps the ring's space holds the shares of W X^T, [kQS][kQT][64][16] (share 0
    // becomes the sum), and the a_t and f_t of the dependent rounds
    static constexpr int q0 = ring;
    static constexpr int part_bytes = kQT * tile_f;
    static constexpr int st = ring + kQS * part_bytes;
    static constexpr int fl = st + kQT * tile_f;
    static constexpr int corr = 0;                                 // (unused)
    static constexpr int total = ring + kQStages * stage_bytes;
};
static_assert(LdsQ::fl + kQT * LdsQ::tile_s <= LdsQ::total && LdsQ::total <= 160 * 1024, "LDS of a gfx950 compute unit");

__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

template <int LOSS, bool OPT = false>
__global__ void __launch_bounds__((kQW + kQL) * kWave) dense_window_shared_kernel(const DenseArgs a, const float *gram, const float *gxt,
                                                                               const float *xq, const float *xu, float *misc,
                                                                               WinPlanD plan, int w0, int nw)
{
    (void)gxt;
    using Lds = LdsQ;
    constexpr int NT = kQW * kWave;                              // working threads
    extern __shared__ __align__(16) char lds[];
    const int d = a.d, K = a.K;
    const int nq = a.R * K;
    const int nblk = (d + 15) / 16;
    const int nstep = (nblk + kQS - 1) / kQS;
    const int npad = (nstep + kQSets * kQStages - 1) / (kQSets * kQStages) * (kQSets * kQStages);   // steps every wavefront walks
    const int q_base = (int)blockIdx.x * kQT * kM;
    const int tid = (int)threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool loader = wave >= kQW;
    const int tau = wave & (kQT - 1), sg = (wave / kQT) & (kQS - 1);
    const int lr = lane & 15, lk = lane >> 4;
    const int q_sw = q_base + tau * kM + lr;                     // this lane's learner in the sweep
    const bool q_ok = q_sw < nq;
    float *vrow = a.V + (int64_t)(q_ok ? q_sw : 0) * d + 4 * lk;
    float *sink = misc + kMiscZeros + (tid & (NT - 1)) * 4;

    // dependent rounds: wavefront m < kQT, lane = 4 learner + quad lane
    float eta = 0.f;
    double sigma0 = 1.0, n2_state = 0.0;
    Hint hint{0.f, 0.f, 0.f};   // optimistic update: carried from round to round, window to window, call to call
    {
        const int q_ch = q_base + wave * kM + (lane >> 2);
        if (wave < kQT && q_ch < nq) {
            eta = a.eta[q_ch % K];
            sigma0 = (double)a.sigma[q_ch];
            n2_state = a.n2[q_ch] * sigma0 * sigma0;
            if (OPT) {
                const int ws0 = plan.start(w0);
                hint.ha = a.ha[q_ch];
                hint.hp = a.hp[q_ch];
                hint.x2p = ws0 == 0 ? a.x2last[0] : a.x2[ws0 - 1];
            }
        }
    }
    auto measured_n2 = [&](int m, int lc) __attribute__((always_inline)) {
        const float *n2s = reinterpret_cast<const float *>(lds + Lds::n2) + m * kQS * 4 * kM;
        double v = 0.0;
#pragma unroll
        for (int i = 0; i < kQS * 4; ++i) v += (double)n2s[i * kM + lc];
        return v;
    };
#ifdef OCO_WIN_PROF
    unsigned long long prof_[8] = {0, 0, 0, 0, 0, 0, 0, 0}, last_ = wall_clock64();
#endif

    // The loader's side of a sweep: rows for (3) from window wu of the piece, rows for (1) from window wq.
    struct Regs { f4 r[6]; };
    Regs rg[kQSets];                                             // loaders: four steps of loads (the prefetch buffer)
    // The loaders' side of a sweep: rows for (3) from window wu of the piece, rows for (1) from window wq.
    // `first`: the loads of the first four steps are issued here; otherwise they were issued at the end of
    // the sweep before (nwu >= 0: issue those of the next sweep, rows from windows nwu / nwq), so that
    // they travel while the dependent rounds run.
    auto load_sweep = [&](int wu, int wq, bool first, int nwu, int nwq) __attribute__((always_inline)) {
        // the learners whose blocks this lane loads, tile by tile
        const float *vr[2];
        bool vok[2];
#pragma unroll
        for (int m = 0; m < 2; ++m) {
            const int q = q_base + (2 * ((wave - kQW) >> 1) + m) * kM + lr;
            vok[m] = q < nq;
            vr[m] = a.V + (int64_t)(vok[m] ? q : 0) * d + 4 * lk;
        }
        // loader j: block kQS s + (j & 1) of step s; j < 2 its rows for (3) and the iterates of tiles 0, 1,
        // j >= 2 its rows for (1) and the iterates of tiles 2, 3
        const int L = (wave - kQW) & 1, part = (wave - kQW) >> 1;
        auto fetch_of = [&](int fu, int fq, int step, Regs &o) __attribute__((always_inline)) {
            const int sc = step < nstep ? step : nstep - 1;
            int blk = sc * kQS + L;
            blk = blk < nblk ? blk : nblk - 1;                   // (rows past the last block: loaded again, not used)
            const float *src = (part == 0 ? xu + ((int64_t)fu * nblk + blk) * kTileFloats
                                          : xq + ((int64_t)fq * nblk + blk) * kTileFloats) + lane * 4;
#pragma unroll
            for (int c = 0; c < 4; ++c) o.r[c] = *reinterpret_cast<const f4 *>(src + c * 256);
            const int vblk = step * kQS + L;
            const bool bok = step < nstep && vblk < nblk && vblk * 16 + 4 * lk < d;
#pragma unroll
            for (int m = 0; m < 2; ++m) o.r[4 + m] = *reinterpret_cast<const f4 *>((bok && vok[m]) ? vr[m] + vblk * 16 : misc);
        };
        auto fetch = [&](int step, Regs &o) __attribute__((always_inline)) { fetch_of(wu, wq, step, o); };
        auto put = [&](int stage, const Regs &o) __attribute__((always_inline)) {
            char *st = lds + Lds::ring + stage * Lds::stage_bytes + lane * 16;
#pragma unroll
            for (int c = 0; c < 4; ++c) *reinterpret_cast<f4 *>(st + L * 8192 + part * 4096 + c * 1024) = o.r[c];
#pragma unroll
            for (int m = 0; m < 2; ++m) *reinterpret_cast<f4 *>(st + Lds::rows_bytes + (L * kQT + 2 * part + m) * 1024) = o.r[4 + m];
        };
        // Phase p (up to barrier p): step p's operands from registers to stage p % 3, then the loads of step
        // p + kQSets into the registers they came from (the registers are the prefetch buffer: four steps of
        // loads are on their way).  After barrier p the working wavefronts read stage p while they work step
        // p - 1; the stage was last read two phases earlier.
        if (first) {
#pragma unroll
            for (int s0 = 0; s0 < kQSets; ++s0) fetch(s0, rg[s0]);
        }
        put(0, rg[0]);
        fetch(kQSets, rg[0]);
        lds_barrier();
        for (int sb = 0; sb < npad; sb += kQSets * kQStages) {
            static_for<kQSets * kQStages>([&](auto uc) __attribute__((always_inline)) {
                constexpr int u = decltype(uc)::value;
                put((u + 1) % kQStages, rg[(u + 1) % kQSets]);
                fetch(sb + u + 1 + kQSets, rg[(u + 1) % kQSets]);
                lds_barrier();
            });
        }
        // (the blocks of iterates of the next sweep's first steps were stored at the start of this one: the
        // working wavefronts have waited for those stores before the last barrier above)
        if (nwu >= 0) {
#pragma unroll
            for (int s0 = 0; s0 < kQSets; ++s0) fetch_of(nwu, nwq, s0, rg[s0]);
        }
        lds_barrier();
        lds_barrier();
        lds_barrier();
    };

    // Labels and Gram table of the next window: the working wavefronts that do not run dependent rounds
    // (kQT .. kQW - 1) load them into registers beside those rounds (whose LDS copies are still in use) and
    // write them to LDS once the rounds are done.
    constexpr int kNPre = (kQW - kQT) * kWave;                  // threads that stage
    constexpr int kGPer = kB * kB / kNPre, kYPer = kQT * kM * kB / kNPre;
    f4 gpre[kGPer / 4];
    float ypre[kYPer];
    float hgpre = 0.f;                                           // (optimistic update: <x_{t-1}, x_t> of one round)
    auto load_next = [&](int wi) __attribute__((always_inline)) {
        const int tp = tid - kQT * kWave;
        const int w = w0 + wi;
        const int ws = plan.start(w), wl = plan.len(w);
        const float *gsrc = gram + (int64_t)wi * kB * kB + tp * kGPer;
#pragma unroll
        for (int i = 0; i < kGPer / 4; ++i) gpre[i] = *reinterpret_cast<const f4 *>(gsrc + 4 * i);
#pragma unroll
        for (int i = 0; i < kYPer; ++i) {
            const int e = tp + i * kNPre, l = e >> 6, t = e & 63;
            const int q = q_base + l;
            const bool ok = a.y && q < nq && t < wl;              // (no label: a zero word)
            ypre[i] = *(ok ? a.y + (int64_t)(q / K) * a.y_run_stride + ws + t : misc);
        }
        if (OPT) hgpre = *((tp < kB && tp < wl) ? a.g01 + ws + tp : misc);
    };
    auto store_next = [&]() __attribute__((always_inline)) {
        const int tp = tid - kQT * kWave;
        double *gd = reinterpret_cast<double *>(lds + Lds::gd);
        const int t = (tp * kGPer) >> 6, t2b = (tp * kGPer) & 63;
#pragma unroll
        for (int i = 0; i < kGPer; ++i) {
            const int t2 = t2b + i;
            const float v = gpre[i >> 2][i & 3];
            gd[(t * 4 + (i & 3)) * kGStride + (t2 >> 2)] = t2 > t ? (double)v : 0.0;
            if (t2 == t) gd[t * 4 * kGStride + 16] = (double)v;
        }
        float *yb = reinterpret_cast<float *>(lds + Lds::yb);
#pragma unroll
        for (int i = 0; i < kYPer; ++i) {
            const int e = tp + i * kNPre, l = e >> 6, t = e & 63;
            yb[((l >> 4) * kB + t) * kM + (l & 15)] = ypre[i];
        }
        if (OPT && tp < kB) reinterpret_cast<float *>(lds + Lds::hg)[tp] = hgpre;
    };

    // The working wavefronts' side.  F and -Bm of this lane's learner (bmr[rs]: round 4 rs + lk); do_q: take
    // the shares of W X^T.  stage_next: first write the staged labels and Gram table to LDS; flush_prev >= 0:
    // write the predictions of window flush_prev to Z.
    auto sweep = [&](auto stager, bool do_q, float F, const float (&bmr)[16], bool stage_next, int flush_prev)
        __attribute__((always_inline)) {
        if (flush_prev >= 0) {
            const int w = w0 + flush_prev;
            const int ws = plan.start(w), wl = plan.len(w);
            const float *zb = reinterpret_cast<const float *>(lds + Lds::zb);
            for (int e = tid; e < kQT * kM * kB; e += NT) {
                const int l = e >> 6, t = e & 63;               // a learner's 64 rounds are contiguous in Z
                const int q = q_base + l;
                if (q < nq && t < wl)
                    a.Z[(int64_t)(q / K) * a.zl.zs_r + (int64_t)(q % K) * a.zl.zs_i + (int64_t)(ws + t) * a.zl.zs_t] =
                        zb[((l >> 4) * kB + t) * kM + (l & 15)];
            }
        }
        if constexpr (decltype(stager)::value) {
            if (stage_next) store_next();
        }
        f4 acc[4];
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) acc[rb] = f4{0.f, 0.f, 0.f, 0.f};
        float nn = 0.f;
        PROF_T(1);
        // Two sets of operand registers: while the matrix instructions of step r - 1 run, the
        // operands of step r come from LDS (the eight wavefronts would otherwise all read right
        // after the barrier, 72 KB through the LDS port with the matrix cores idle).
        struct In { f4 xu[4], xq[4], vb; };
        In in[2];
        auto read_stage = [&](int stage, In &o) __attribute__((always_inline)) {
            const char *stg = lds + Lds::ring + stage * Lds::stage_bytes;
            const char *rows = stg + sg * 8192 + lane * 16;
            o.vb = *reinterpret_cast<const f4 *>(stg + Lds::rows_bytes + (sg * kQT + tau) * 1024 + lane * 16);
#pragma unroll
            for (int c = 0; c < 4; ++c) o.xu[c] = *reinterpret_cast<const f4 *>(rows + c * 1024);
#pragma unroll
            for (int c = 0; c < 4; ++c) o.xq[c] = *reinterpret_cast<const f4 *>(rows + 4096 + c * 1024);
        };
        lds_barrier();                                           // the loader has stage 0 complete
        read_stage(0, in[0]);
        for (int sb = 0; sb < npad; sb += 2 * kQStages) {
            static_for<2 * kQStages>([&](auto uc) __attribute__((always_inline)) {
                constexpr int u = decltype(uc)::value;
                const int step = sb + u;
                const int blk = step * kQS + sg;
                // all but the seven youngest stores have been acknowledged: among them those of the first four
                // steps (npad >= 12), which the loaders read again right after this barrier
                if (step == npad - 1) asm volatile("s_waitcnt vmcnt(7)" ::: "memory");
                lds_barrier();                                   // stage step + 1 complete, own reads of stage step done
                read_stage((u + 1) % kQStages, in[(u + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
                const bool active = step < nstep && blk < nblk;  // wavefront-uniform
                if (active) {
                    In &c = in[u & 1];
                    f4 vb = c.vb;
                    f4 vo = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int r = 0; r < 4; ++r) vb[r] *= F;
#pragma unroll
                    for (int rs = 0; rs < 16; rs += 2) {
                        vb = __builtin_amdgcn_mfma_f32_16x16x4f32(c.xu[rs >> 2][rs & 3], bmr[rs], vb, 0, 0, 0);
                        vo = __builtin_amdgcn_mfma_f32_16x16x4f32(c.xu[rs >> 2][(rs & 3) + 1], bmr[rs + 1], vo, 0, 0, 0);
                    }
#pragma unroll
                    for (int r = 0; r < 4; ++r) vb[r] += vo[r];
#pragma unroll
                    for (int r = 0; r < 4; ++r) nn = fmaf(vb[r], vb[r], nn);
                    {
                        const bool ok = q_ok && blk * 16 + 4 * lk < d;
                        float *dst = ok ? vrow + blk * 16 : sink;
                        *reinterpret_cast<f4 *>(dst) = vb;
                    }
                    if (do_q) {
#pragma unroll
                        for (int r = 0; r < 4; ++r)
#pragma unroll
                            for (int rb = 0; rb < 4; ++rb)
                                acc[rb] = __builtin_amdgcn_mfma_f32_16x16x4f32(c.xq[rb][r], vb[r], acc[rb], 0, 0, 0);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            });
        }
        PROF_T(2);
        lds_barrier();                                           // every wavefront is done with the ring
        {
            float *part = reinterpret_cast<float *>(lds + Lds::q0 + sg * Lds::part_bytes + tau * Lds::tile_f);
#pragma unroll
            for (int rb = 0; rb < 4; ++rb)
#pragma unroll
                for (int r = 0; r < 4; ++r) part[(rb * 16 + 4 * lk + r) * kM + lr] = acc[rb][r];
            reinterpret_cast<float *>(lds + Lds::n2)[(tau * kQS * 4 + sg * 4 + lk) * kM + lr] = nn;
        }
        lds_barrier();
        // the two shares of every tile's W X^T, summed in place
        if (do_q) {
            float *p0 = reinterpret_cast<float *>(lds + Lds::q0);
            const float *p1 = reinterpret_cast<const float *>(lds + Lds::q0 + Lds::part_bytes);
#pragma unroll
            for (int i = 0; i < kQT * kB * kM / NT; ++i) p0[tid + i * NT] += p1[tid + i * NT];
        }
        lds_barrier();
        PROF_T(3);
    };

    // Three programs with the same sequence of barriers, one per kind of wavefront, so that what one kind
    // keeps in registers across the window loop (the loaders' prefetch buffer, the staged inputs, the state of
    // the dependent rounds) is not live in the code of the others.
    // CHAIN: wavefronts 0 .. kQT - 1 run the dependent rounds of their tile; the other working wavefronts
    // stage the next window's labels and Gram table meanwhile.
    auto worker = [&](auto chain_tag) __attribute__((always_inline)) {
        constexpr bool CHAIN = decltype(chain_tag)::value;
        using Stager = std::integral_constant<bool, !CHAIN>;
        {
            // the stored iterates times the rows of the first window: a sweep whose step changes nothing
            float zero[16];
#pragma unroll
            for (int i = 0; i < 16; ++i) zero[i] = 0.f;
            if constexpr (!CHAIN) load_next(0);
            sweep(Stager{}, true, 1.f, zero, true, -1);
        }
        for (int k = 0; k < nw; ++k) {
            const bool more = k + 1 < nw;
            if constexpr (CHAIN) {
                double n2 = k == 0 ? n2_state : measured_n2(wave, lane >> 2);
                const double scale = k == 0 ? sigma0 : 1.0;
                bool projected;
                (void)chain_window<LOSS, Lds, OPT>(lds, 0, wave, lane, plan.len(w0 + k), eta, (double)a.D, scale, scale, n2, projected,
                                                   &hint);
            } else {
                if (more) load_next(k + 1);
            }
            PROF_T(0);
            // the iterates the last sweep stored are read by the loaders in the next one
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            lds_barrier();
            PROF_T(4);
            float bmr[16];
            const float *bml = reinterpret_cast<const float *>(lds + Lds::bm + tau * Lds::tile_f);
#pragma unroll
            for (int rs = 0; rs < 16; ++rs) bmr[rs] = bml[(rs * 4 + lk) * kM + lr];
            const float F = reinterpret_cast<const float *>(lds + Lds::fv)[tau * kM + lr];
            sweep(Stager{}, more, F, bmr, more, k);
        }
    };
    if (loader) {
        load_sweep(0, 0, true, 0, nw > 1 ? 1 : 0);
        for (int k = 0; k < nw; ++k) {
            const bool more = k + 1 < nw;
            lds_barrier();
            load_sweep(k, more ? k + 1 : k, false, more ? k + 1 : -1, k + 2 < nw ? k + 2 : k + 1);
        }
    } else if (wave < kQT) {
        worker(std::true_type{});
    } else {
        worker(std::false_type{});
    }
#ifdef OCO_WIN_PROF
    if (threadIdx.x == 0 && blockIdx.x == 0)
        for (int i = 0; i < 8; ++i) g_win_prof[i] = prof_[i];
#endif
    // ---- state out: the iterates themselves (scale 1) and their squared norms ----------------------
    {
        const int q_ch = q_base + wave * kM + (lane >> 2);
        if (wave < kQT && (lane & 3) == 0 && q_ch < nq) {
            a.sigma[q_ch] = 1.f;
            a.n2[q_ch] = measured_n2(wave, lane >> 2);
            if (OPT) { a.ha[q_ch] = hint.ha; a.hp[q_ch] = hint.hp; }
        }
    }
}

using WindowKernel = void (*)(const DenseArgs, const float *, const float *, const float *, const float *, float *, WinPlanD, int,
                              int);

// mode 0: iterates in registers (8 wavefronts, one tile); 1: streamed, two tiles per workgroup
// (8 wavefronts); 2: streamed, one tile, 16 wavefronts; 3: four tiles, loading wavefronts; 4: iterates
// of two tiles in registers (8 wavefronts, d <= 1024)
// (opt: the optimistic update, built into the three kernels the launcher picks by itself)
template <int LOSS> WindowKernel pick_window_kernel(int nblk, int mode, bool opt, int *waves, int *tiles, int *lds_bytes)
{
    if (mode == 4) {
        *waves = kNW8; *tiles = 2; *lds_bytes = LdsT<kNW8, 2>::total;
        if (opt) return dense_window_kernel<LOSS, 9, true, kNW8, 2, true>;
        return dense_window_kernel<LOSS, 9, true, kNW8, 2>;
    }
    if (opt) {
        if (mode == 3) {
            *waves = kQW + kQL; *tiles = kQT; *lds_bytes = LdsQ::total;
            return dense_window_shared_kernel<LOSS, true>;
        }
        *waves = kNW8; *tiles = 2; *lds_bytes = LdsT<kNW8, 2>::total;
        return dense_window_kernel<LOSS, 1, false, kNW8, 2, true>;
    }
    if (mode == 0) {
        *waves = kNW8; *tiles = 1; *lds_bytes = LdsT<kNW8, 1>::total;
        if (nblk <= 8 * kNW8) return dense_window_kernel<LOSS, 8, true, kNW8, 1>;
        return dense_window_kernel<LOSS, 32, true, kNW8, 1>;
    }
    if (mode == 1) {
        *waves = kNW8; *tiles = 2; *lds_bytes = LdsT<kNW8, 2>::total;
        return dense_window_kernel<LOSS, 1, false, kNW8, 2>;
    }
    if (mode == 3) {
        *waves = kQW + kQL; *tiles = kQT; *lds_bytes = LdsQ::total;
        return dense_window_shared_kernel<LOSS>;
    }
    *waves = kNW16; *tiles = 1; *lds_bytes = LdsT<kNW16, 1>::total;
    return dense_window_kernel<LOSS, 1, false, kNW16, 1>;
}

// scratch: Gram and cross Gram matrices of the windows of a piece, then the two tiled copies of its rows
struct Scratch {
    int64_t piece_windows;      // windows per launch
    size_t gram_floats, tile_floats;
    size_t total_floats() const { return 2 * gram_floats + 2 * tile_floats + kMiscFloats; }
};
Scratch scratch_layout(int64_t n_max, int64_t d)
{
    const int64_t nblk = (d + 15) / 16;
    const int64_t win_bytes = nblk * kTileFloats * (int64_t)sizeof(float);
    Scratch sc;
    sc.piece_windows = std::max<int64_t>(1, std::min<int64_t>(kPieceBytes / win_bytes, n_max / kB + 2));
    sc.gram_floats = (size_t)sc.piece_windows * kB * kB;
    sc.tile_floats = (size_t)sc.piece_windows * nblk * kTileFloats;
    return sc;
}

}  // namespace

#ifdef OCO_WIN_PROF
extern "C" int oco_debug_win_prof(unsigned long long *out)
{
    return (int)hipMemcpyFromSymbol(out, HIP_SYMBOL(g_win_prof), sizeof(unsigned long long) * 8);
}
#endif

size_t dense_gram_bytes(int64_t n_max, int64_t d) { return scratch_layout(n_max, d).total_floats() * sizeof(float); }

bool dense_window_supported(const DenseArgs &a)
{
    // a shared stream whose rows can be read 16 bytes at a time
    return a.x_shared && a.vec_ok && a.gram != nullptr;
}

bool dense_window_wanted(const DenseArgs &a)
{
    if (!dense_window_supported(a)) return false;
    const int64_t path = a.tune->get(OCO_OPT_DENSE_PATH);
    if (path == 1) return a.d > 64 * kWave;                     // the register kernel cannot hold more
    if (path == 2) return true;
    // measured on MI355X: c4 (16384 learners, d = 4096) 72 ms against the register kernel's 136 ms; c3 (4352
    // learners, d = 1000) 50 ms against 62 ms.  Narrower problems and fewer learners stay with the register
    // kernel (a round of the dependent rounds here costs about 0.4 us per tile whatever d is).
    return a.d > 64 * kWave || ((int64_t)a.R * a.K >= 2048 && a.d >= 512);
}

hipError_t launch_dense_window(const DenseArgs &a0, int loss, hipStream_t s, const PieceHook *hook)
{
    DenseArgs a = a0;
    if (a.n <= 0) return hipSuccess;
    if (!dense_window_supported(a)) return hipErrorInvalidValue;
    const WinPlanD plan{a.t0, a.n};
    const int nwin = plan.count();
    const int nblk = (a.d + 15) / 16;
    const Scratch sc = scratch_layout(a.n_max, a.d);
    float *gram = a.gram, *gxt = gram + sc.gram_floats, *xq = gxt + sc.gram_floats, *xu = xq + sc.tile_floats;
    float *misc = xu + sc.tile_floats;
    {
        ComparatorGemmArgs g{};
        g.x = a.x; g.u = a.u; g.seg_start = a.seg_start; g.S = a.S; g.Z = a.Z; g.zl = a.zl;
        g.d = a.d; g.K = a.K; g.R = a.R; g.t0 = a.t0; g.n = a.n; g.vec_ok = a.vec_ok;
        hipError_t e = launch_comparator_gemm(g, s);
        if (e != hipSuccess) return e;
    }
    if (a.optimistic) {
        // ||x_t||^2 and <x_{t-1}, x_t> of the call's rounds (the first against the row kept from the call before)
        hipError_t e = launch_hint_scalars(a, s);
        if (e != hipSuccess) return e;
    }
    // where the iterates live: OCO_OPT_WINDOW_RESIDENT 1 registers (d <= 4096), 0 streamed (two tiles per
    // workgroup), 2 streamed (one tile, sixteen wavefronts), 3 streamed with loading wavefronts (four tiles),
    // 4 registers, two tiles per workgroup (d <= 1024).
    // Unset: streamed, two tiles -- on c4 as fast as the registers (every round row a wavefront loads
    // serves two tiles), on c3 half as many workgroups --, two tiles in registers where they fit and the
    // wavefronts have several blocks each (c3: 41.8 against 46.4 ms), or, with at least four tiles per compute unit's
    // workgroup on every one of 256 compute units and wide rows, the loading wavefronts (c4: 67.4 against
    // 70.4 ms; c3, bound by the dependent rounds, which that kernel does not overlap: 101 against 47.5 ms).
    const int64_t ropt = a.tune->get(OCO_OPT_WINDOW_RESIDENT);
    const bool fits = a.d <= 16 * kNW8 * 32;
    const bool many = (int64_t)a.R * a.K >= 1024 * kM && nblk >= 128;
    const bool fits2 = a.d <= 16 * kNW8 * 8;
    int mode = (ropt == 1 && fits) ? 0 : ropt == 2 ? 2 : (ropt == 3 || (ropt < 0 && many)) ? 3
               : ((ropt == 4 || (ropt < 0 && nblk >= 32)) && fits2) ? 4 : 1;
    if (a.optimistic && mode != 3 && mode != 4) mode = 1;    // (the optimistic update: three of the kernels only)
    const bool resident = mode == 0 || mode == 4;
    if (a.tune->get(OCO_OPT_VERBOSE) == 1)
        fprintf(stderr, "dense plan: windowed contraction kernel, %d windows in pieces of %lld, %d tiles, iterates %s\n",
                nwin, (long long)sc.piece_windows, (a.R * a.K + kM - 1) / kM,
                mode == 4 ? "in registers, two tiles per workgroup" : resident ? "in registers" : mode == 1 ? "streamed from HBM, two tiles per workgroup"
                : mode == 3 ? "streamed from HBM, four tiles per workgroup, rows through LDS" : "streamed from HBM");
    WindowKernel kern = nullptr;
    int waves = 0, tiles = 1, lds_bytes = 0;
    switch (loss) {
        case 0: kern = pick_window_kernel<0>(nblk, mode, a.optimistic != 0, &waves, &tiles, &lds_bytes); break;
        case 1: kern = pick_window_kernel<1>(nblk, mode, a.optimistic != 0, &waves, &tiles, &lds_bytes); break;
        case 2: kern = pick_window_kernel<2>(nblk, mode, a.optimistic != 0, &waves, &tiles, &lds_bytes); break;
        default: return hipErrorInvalidValue;
    }
    const int ntiles = (a.R * a.K + kM * tiles - 1) / (kM * tiles);   // workgroups
    // The caller's work on a piece's rounds (the meta kernel) goes beside the window kernel of the following
    // piece where that leaves a quarter of the compute units or more without a workgroup (c3: 136 of 256;
    // 46.7 -> 45.8 ms per step: the window kernel is slower beside it, 6.25 against 5.72 ms per launch.
    // Handed over only behind the following piece's pre-passes: 46.2 ms).
    int ncu = 256;
    {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            ncu <= 0)
            ncu = 256;
    }
    const bool beside = hook && hook->fn && 4 * (int64_t)ntiles <= 3 * (int64_t)ncu;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                       lds_bytes);
    if (e != hipSuccess) return e;
    for (int w0 = 0; w0 < nwin; w0 += (int)sc.piece_windows) {
        const int nw = std::min<int>((int)sc.piece_windows, nwin - w0);
        hipLaunchKernelGGL(dense_tile_kernel, dim3((unsigned)nblk, (unsigned)nw), dim3(64), 0, s, a.x, a.d, plan, w0, xq, xu, misc);
        hipLaunchKernelGGL(dense_gram_kernel, dim3((unsigned)nw), dim3(512), 0, s, xq, nblk, gram, gxt);
        e = clock_begin(a.clock, s, mode == 3 ? "dense_window_shared_kernel" : "dense_window_kernel");
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(kern, dim3((unsigned)ntiles), dim3(waves * kWave), lds_bytes, s, a, gram, gxt, xq, xu, misc, plan, w0, nw);
        e = hipGetLastError();
        if (e == hipSuccess) e = clock_end(a.clock, s);
        if (e == hipSuccess && beside) {
            const int off = plan.start(w0), end = plan.start(w0 + nw - 1) + plan.len(w0 + nw - 1);
            e = hook->fn(hook->ctx, off, end - off);
        }
        if (e != hipSuccess) return e;
    }
    return a.optimistic ? launch_keep_last_row(a, s) : hipSuccess;
}

}  // namespace oco
