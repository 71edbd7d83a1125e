// Host side of the C ABI declared in include/oco.h: argument validation,
// workspace layout, kernel sequencing.  No device memory is allocated here.
#include "../../include/oco.h"
#include "oco_internal.h"

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

using namespace oco;

namespace {

size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Layout {
    size_t off_V = 0, off_sigma = 0, off_n2 = 0, off_L = 0, off_last = 0, off_regret = 0, off_eta = 0,
           off_seg = 0, off_Z = 0, off_X2 = 0, off_gram = 0, total = 0;
    size_t off_ha = 0, off_hp = 0, off_xlast = 0, off_x2last = 0, off_G01 = 0;   // optimistic mode only
    size_t off_lastcol = 0, off_lastval = 0;                                       // optimistic + sparse
    size_t state_bytes = 0;   // [off_V, off_V + state_bytes) is zeroed by reset (V, sigma, n2, L, regret)
    int64_t n_sigma = 0;
    int RKp = 0;
    int64_t n_max = 0;
};

bool finite_pos(double v) { return std::isfinite(v) && v > 0.0; }

// Returns OCO_OK and fills `lay`, or the status that describes what is wrong with cfg.
int validate_and_layout(const oco_config *c, Layout *lay)
{
    if (!c || !c->eta) return OCO_EINVAL;
    if (c->d <= 0 || c->K <= 0 || c->T <= 0 || c->R <= 0) return OCO_EINVAL;
    if (c->optimistic < 0 || c->optimistic > 2 || c->n_max < 0) return OCO_EINVAL;
    if (!finite_pos(c->D) || !finite_pos(c->G) || !std::isfinite(c->eps) || c->eps < 0.0) return OCO_EINVAL;
    if (c->loss < OCO_LINEAR || c->loss > OCO_LOGISTIC) return OCO_EINVAL;
    if (c->x_shared != 0 && c->x_shared != 1) return OCO_EINVAL;
    if (c->sparse_nnz < 0) return OCO_EINVAL;
    if (c->K > OCO_MAX_K) return OCO_EUNSUPPORTED;
    for (int64_t i = 0; i < c->K; ++i)
        if (!finite_pos(c->eta[i])) return OCO_EINVAL;
    if (c->d > INT32_MAX || c->T > INT32_MAX || c->R > (1 << 24)) return OCO_EUNSUPPORTED;
    const int64_t n_max = c->n_max == 0 ? c->T : (c->n_max < c->T ? c->n_max : c->T);
    const int64_t RK = c->R * c->K;
    if (RK > (1 << 26)) return OCO_EUNSUPPORTED;
    if (c->sparse_nnz > 0) {
        if (c->sparse_nnz > OCO_MAX_NNZ || c->sparse_nnz > c->d) return OCO_EUNSUPPORTED;
        if (!c->x_shared) return OCO_EUNSUPPORTED;
    } else if (!dense_supported(c->d, c->x_shared)) {
        return OCO_EUNSUPPORTED;
    } else if (c->d > 4096 && c->d % 4 != 0) {
        return OCO_EUNSUPPORTED;      // beyond one wavefront's registers only the windowed kernel runs
    }
    Layout l;
    l.n_max = n_max;
    size_t off = 0;
    l.off_V = off;
    if (c->sparse_nnz > 0) {
        // row length of V: the learners padded to whole wavefronts, plus 32 floats, which makes
        // it an odd number of 128-byte lines.  A workgroup touches the same few bytes of many rows;
        // with a power-of-two row length all of them would sit in one L2 channel.
        l.RKp = (int)align_up((size_t)RK, kWave) + 32;
        off += align_up(sizeof(float) * (size_t)c->d * l.RKp, 256);
        l.off_sigma = off; l.n_sigma = l.RKp;
        off += align_up(sizeof(double) * l.RKp, 256);
        l.off_n2 = off;
        off += align_up(sizeof(double) * l.RKp, 256);
    } else {
        off += align_up(sizeof(float) * (size_t)RK * c->d, 256);
        l.off_sigma = off; l.n_sigma = RK;
        off += align_up(sizeof(float) * (size_t)RK, 256);
        l.off_n2 = off;
        off += align_up(sizeof(double) * (size_t)RK, 256);
    }
    l.off_L = off;       off += align_up(sizeof(double) * (size_t)RK, 256);
    l.off_regret = off;  off += align_up(sizeof(double) * (size_t)c->R, 256);
    if (c->optimistic == 2) {                              // the meta learner's hint: last observed losses
        l.off_last = off;
        off += align_up(sizeof(double) * (size_t)RK, 256);
    }
    if (c->optimistic && c->sparse_nnz > 0) {
        l.off_ha = off;      off += align_up(sizeof(float) * (size_t)l.RKp, 256);
        l.off_hp = off;      off += align_up(sizeof(float) * (size_t)l.RKp, 256);
        l.off_x2last = off;  off += align_up(sizeof(float) * (size_t)l.RKp, 256);
        l.off_lastcol = off; off += align_up(sizeof(int32_t) * OCO_MAX_NNZ, 256);
        l.off_lastval = off; off += align_up(sizeof(float) * OCO_MAX_NNZ, 256);
        l.off_xlast = off;   off += align_up(sizeof(float) * (size_t)c->d, 256);
    } else if (c->optimistic) {
        const size_t nx = c->x_shared ? 1 : (size_t)c->R;
        l.off_ha = off;      off += align_up(sizeof(float) * (size_t)RK, 256);
        l.off_hp = off;      off += align_up(sizeof(float) * (size_t)RK, 256);
        l.off_xlast = off;   off += align_up(sizeof(float) * nx * (size_t)c->d, 256);
        l.off_x2last = off;  off += align_up(sizeof(float) * nx, 256);
    }
    l.state_bytes = off;
    l.off_eta = off;     off += align_up(sizeof(float) * (size_t)c->K, 256);
    l.off_seg = off;     off += align_up(sizeof(int64_t) * OCO_MAX_SEGMENTS, 256);
    l.off_Z = off;       off += align_up(sizeof(float) * (size_t)c->R * (c->K + 1) * align_up(n_max, 64), 256);
    if (c->sparse_nnz == 0) {
        l.off_X2 = off;
        off += align_up(sizeof(float) * (size_t)(c->x_shared ? 1 : c->R) * align_up(n_max, 64), 256);
        if (c->optimistic) {
            l.off_G01 = off;
            off += align_up(sizeof(float) * (size_t)(c->x_shared ? 1 : c->R) * align_up(n_max, 64), 256);
        }
        if (c->x_shared) {
            l.off_gram = off;
            off += align_up(dense_gram_bytes(n_max, c->d), 256);
        }
    } else {
        l.off_gram = off;
        off += align_up(sparse_scratch_bytes(n_max), 256);
    }
    l.total = off;
    *lay = l;
    return OCO_OK;
}

}  // namespace

struct oco_state {
    oco_config cfg;
    double eta[OCO_MAX_K];
    int64_t seg_start[OCO_MAX_SEGMENTS];
    Layout lay;
    char *ws = nullptr;
    hipStream_t stream = nullptr;
    const float *u_dev = nullptr;
    int64_t S = 0;
    int64_t t_done = 0;
    bool failed = false;       // a HIP error hit a call half-way: the device state is undefined until oco_reset
    bool is_static = false;    // created by oco_create_static: no second stream, no events
    bool timing = false, timed = false;
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    LaunchClock clock;         // events exist once timing has been switched on
    Tuning tune;
    DensePlanCache dense_plan;
    // The meta kernel of a piece of a call depends on that piece's predictions only, and no
    // round kernel depends on a meta kernel (every base learner steps at its own iterate): it
    // runs on a second stream beside the round kernels of the following pieces, and the
    // caller's stream waits for it at the end of the call.
    hipStream_t side = nullptr;
    std::vector<hipEvent_t> piece_ev;
    hipEvent_t join_ev = nullptr;

    ~oco_state() {
        for (auto e : ev) if (e) (void)hipEventDestroy(e);
        for (auto e : clock.ev) if (e) (void)hipEventDestroy(e);
        for (auto e : piece_ev) if (e) (void)hipEventDestroy(e);
        if (join_ev) (void)hipEventDestroy(join_ev);
        if (side) { (void)hipStreamSynchronize(side); (void)hipStreamDestroy(side); }
    }
    template <class T> T *at(size_t off) const { return reinterpret_cast<T *>(ws + off); }
    ZLayout zlayout() const {
        const int64_t nz = (int64_t)align_up((size_t)lay.n_max, 64);
        if (cfg.sparse_nnz > 0) return ZLayout{cfg.K + 1, 1, cfg.R * (cfg.K + 1)};
        return ZLayout{(cfg.K + 1) * nz, nz, 1};
    }
};

namespace {

// Workspace of oco_create_static: part of the library's image, one copy per GPU.  In host code
// the array's name only stands for the symbol; the device address comes from
// hipGetSymbolAddress, once per device, and only that pointer is ever handed to kernels.
__device__ __align__(256) unsigned char scratch[OCO_STATIC_WS_BYTES];
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];      // per device; null until looked up
std::mutex g_scratch_mu;

// Device address of this GPU's copy of `scratch` (null on error).
void *static_workspace()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

// Common part of oco_create and oco_create_static: `side_stream` says whether the state gets a
// second stream (and the event that joins it) for work beside the round kernels.
int create_on(const oco_config *cfg, const Layout &l, void *dev_ws, void *hip_stream, bool side_stream,
              oco_state **out)
{
    oco_state *st = new (std::nothrow) oco_state();
    if (!st) return OCO_ENOMEM;
    st->cfg = *cfg;
    for (int64_t i = 0; i < cfg->K; ++i) st->eta[i] = cfg->eta[i];
    st->cfg.eta = st->eta;
    st->lay = l;
    st->ws = static_cast<char *>(dev_ws);
    st->stream = static_cast<hipStream_t>(hip_stream);
    st->is_static = !side_stream;
    if (side_stream &&
        (hipStreamCreateWithFlags(&st->side, hipStreamNonBlocking) != hipSuccess ||
         hipEventCreateWithFlags(&st->join_ev, hipEventDisableTiming) != hipSuccess)) {
        delete st;
        return OCO_EHIP;
    }
    int rc = oco_reset(st);
    if (rc != OCO_OK) { delete st; return rc; }
    *out = st;
    return OCO_OK;
}

}  // namespace

extern "C" {

int oco_step_grid(double D, double G, int64_t T, int64_t K, double *out)
{
    if (!out || K <= 0 || T <= 0 || !finite_pos(D) || !finite_pos(G)) return OCO_EINVAL;
    const double base = D / (G * std::sqrt((double)T));
    for (int64_t i = 0; i < K; ++i) out[i] = std::ldexp(base, (int)i);
    return OCO_OK;
}

int64_t oco_paper_num_learners(int64_t T)
{
    if (T <= 0) return OCO_EINVAL;
    return (int64_t)std::ceil(0.5 * std::log2(1.0 + (double)T)) + 1;
}

size_t oco_workspace_bytes(const oco_config *cfg)
{
    Layout l;
    return validate_and_layout(cfg, &l) == OCO_OK ? l.total : 0;
}

int oco_reset(oco_state *st)
{
    if (!st) return OCO_EINVAL;
    hipError_t e = launch_init_state(st->at<void>(st->lay.off_V), st->lay.state_bytes,
                                     st->at<void>(st->lay.off_sigma), st->lay.n_sigma,
                                     st->cfg.sparse_nnz > 0, st->stream);
    if (e != hipSuccess) return OCO_EHIP;
    // the step sizes travel as a kernel argument (no host buffer has to outlive the call)
    EtaTable tab;
    for (int64_t i = 0; i < OCO_MAX_K; ++i) tab.v[i] = i < st->cfg.K ? (float)st->eta[i] : 0.f;
    if (launch_set_eta(st->at<float>(st->lay.off_eta), tab, (int)st->cfg.K, st->stream) != hipSuccess)
        return OCO_EHIP;
    st->t_done = 0;
    st->failed = false;
    return OCO_OK;
}

int oco_create(const oco_config *cfg, void *dev_ws, size_t ws_bytes, void *hip_stream, oco_state **out)
{
    if (!out) return OCO_EINVAL;
    *out = nullptr;
    Layout l;
    int rc = validate_and_layout(cfg, &l);
    if (rc != OCO_OK) return rc;
    if (!dev_ws || (reinterpret_cast<uintptr_t>(dev_ws) & 255u)) return OCO_EINVAL;
    if (ws_bytes < l.total) return OCO_ENOMEM;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) return OCO_EHIP;
    return create_on(cfg, l, dev_ws, hip_stream, true, out);
}

int oco_create_static(const oco_config *cfg, void *hip_stream, oco_state **out)
{
    if (!out) return OCO_EINVAL;
    *out = nullptr;
    Layout l;
    int rc = validate_and_layout(cfg, &l);
    if (rc != OCO_OK) return rc;
    if (l.total > (size_t)OCO_STATIC_WS_BYTES) return OCO_ENOMEM;
    int ndev = 0;
    if (hipGetDeviceCount(&ndev) != hipSuccess || ndev <= 0) return OCO_EHIP;
    void *ws = static_workspace();
    if (!ws) return OCO_EHIP;
    return create_on(cfg, l, ws, hip_stream, false, out);
}

int oco_set_option(oco_state *st, int key, int64_t value)
{
    if (!st || key < 0 || key >= OCO_OPT_COUNT || value < -1) return OCO_EINVAL;
    bool ok = true;
    switch (key) {
        case OCO_OPT_META_BESIDE: case OCO_OPT_COMPARATOR_GEMM: case OCO_OPT_DENSE_HALF:
        case OCO_OPT_SPARSE_PIPE: case OCO_OPT_VERBOSE: case OCO_OPT_SPARSE_FETCH:
            ok = value <= 1; break;
        case OCO_OPT_WINDOW_RESIDENT: ok = value <= 4; break;
        case OCO_OPT_DENSE_PATH:
            ok = value == -1 || value == 1 || value == 2;
            if (value == 2 && (st->cfg.sparse_nnz > 0 || !st->cfg.x_shared || st->cfg.d % 4 != 0))
                return OCO_EUNSUPPORTED;
            if (value == 1 && st->cfg.sparse_nnz == 0 && st->cfg.d > 4096) return OCO_EUNSUPPORTED;
            break;
        case OCO_OPT_DENSE_WPB: ok = value == -1 || (value >= 1 && value <= 16); break;
        case OCO_OPT_DENSE_PIECES: ok = value == -1 || (value >= 1 && value <= (1 << 20)); break;
        case OCO_OPT_SPARSE_LPW:
            ok = value == -1 || value == 4 || value == 8 || value == 16 || value == 32 || value == 64; break;
        default: ok = false;
    }
    if (!ok) return OCO_EINVAL;
    st->tune.v[key] = value;
    st->dense_plan.valid = false;
    return OCO_OK;
}

int oco_set_comparator(oco_state *st, const float *u_dev, const int64_t *seg_start_host, int64_t S)
{
    if (!st || !u_dev || !seg_start_host || S <= 0) return OCO_EINVAL;
    if (S > OCO_MAX_SEGMENTS) return OCO_ERANGE;
    if (reinterpret_cast<uintptr_t>(u_dev) & 15u) return OCO_EINVAL;
    if (seg_start_host[0] != 0) return OCO_EINVAL;
    for (int64_t s = 1; s < S; ++s)
        if (seg_start_host[s] <= seg_start_host[s - 1]) return OCO_EINVAL;
    std::memcpy(st->seg_start, seg_start_host, sizeof(int64_t) * (size_t)S);
    if (hipMemcpyAsync(st->at<int64_t>(st->lay.off_seg), st->seg_start, sizeof(int64_t) * S,
                       hipMemcpyHostToDevice, st->stream) != hipSuccess)
        return OCO_EHIP;
    // the host copy may be rewritten by a later call: make sure the transfer has left it
    if (hipStreamSynchronize(st->stream) != hipSuccess) return OCO_EHIP;
    st->u_dev = u_dev;
    st->S = S;
    return OCO_OK;
}

int oco_run_rounds(oco_state *st, const oco_rounds *rd, int64_t t0, int64_t n)
{
    if (!st || !rd || n < 0 || t0 < 0) return OCO_EINVAL;
    if (st->failed) return OCO_EHIP;
    if (t0 != st->t_done) return OCO_ESEQ;
    if (t0 + n > st->cfg.T || n > st->lay.n_max) return OCO_ERANGE;
    if (!st->u_dev) return OCO_ENOCOMP;
    if (n == 0) return OCO_OK;
    const oco_config &c = st->cfg;
    const bool sparse = c.sparse_nnz > 0;
    if (sparse ? (!rd->col || !rd->val) : !rd->x) return OCO_EINVAL;
    if (c.loss != OCO_LINEAR && !rd->y) return OCO_EINVAL;
    if (rd->x_run_stride < 0 || rd->y_run_stride < 0) return OCO_EINVAL;
    const int64_t xrs = rd->x_run_stride ? rd->x_run_stride : n * c.d;
    const int64_t yrs = rd->y_run_stride ? rd->y_run_stride : n;
    if (!sparse && !c.x_shared && xrs < n * c.d) return OCO_EINVAL;
    if (rd->y && yrs < n) return OCO_EINVAL;
    auto mis = [](const void *p, unsigned a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; };
    if (mis(rd->x, 4) || mis(rd->y, 4) || mis(rd->col, 4) || mis(rd->val, 4)) return OCO_EINVAL;
    if (!sparse && c.d > 4096 && mis(rd->x, 16)) return OCO_EUNSUPPORTED;

    const Layout &l = st->lay;
    const ZLayout zl = st->zlayout();
    hipError_t e;
    if (st->timing && hipEventRecord(st->ev[0], st->stream) != hipSuccess) return OCO_EHIP;
    st->clock.launches = st->clock.timed = 0;
    // from here on part of the call's work may be on the device when an error comes back
    auto fail = [st]() { st->failed = true; return (int)OCO_EHIP; };

    // Meta kernel of the rounds [off, off + len) of this call, on the second stream.
    struct MetaPipe {
        oco_state *st; MetaArgs m; int loss; size_t used = 0;
        // the second stream waits for what is on the call's stream now
        hipError_t follow() {
            if (used == st->piece_ev.size()) {
                hipEvent_t ev;
                hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
                if (e != hipSuccess) return e;
                try {
                    st->piece_ev.push_back(ev);          // nothing may throw across the C boundary
                } catch (...) {
                    (void)hipEventDestroy(ev);
                    return hipErrorOutOfMemory;
                }
            }
            hipEvent_t ev = st->piece_ev[used++];
            hipError_t e = hipEventRecord(ev, st->stream);
            if (e == hipSuccess) e = hipStreamWaitEvent(st->side, ev, 0);
            return e;
        }
        static hipError_t beside(void *ctx, hipStream_t *out) {
            MetaPipe &p = *static_cast<MetaPipe *>(ctx);
            *out = p.st->side;
            return p.follow();
        }
        static hipError_t piece(void *ctx, int off, int len) {
            MetaPipe &p = *static_cast<MetaPipe *>(ctx);
            oco_state *st = p.st;
            hipError_t e = p.follow();
            if (e != hipSuccess) return e;
            MetaArgs m = p.m;
            m.Z += (int64_t)off * m.zl.zs_t;
            if (m.y) m.y += off;
            m.n = len;
            return launch_meta(m, p.loss, st->side);
        }
        // an event of the pool, recorded on the second stream / waited for by the call's stream
        hipEvent_t marked = nullptr;
        static hipError_t mark(void *ctx) {
            MetaPipe &p = *static_cast<MetaPipe *>(ctx);
            oco_state *st = p.st;
            if (p.used == st->piece_ev.size()) {
                hipEvent_t ev;
                hipError_t e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
                if (e != hipSuccess) return e;
                try {
                    st->piece_ev.push_back(ev);
                } catch (...) {
                    (void)hipEventDestroy(ev);
                    return hipErrorOutOfMemory;
                }
            }
            p.marked = st->piece_ev[p.used++];
            return hipEventRecord(p.marked, st->side);
        }
        static hipError_t wait_mark(void *ctx) {
            MetaPipe &p = *static_cast<MetaPipe *>(ctx);
            if (!p.marked) return hipSuccess;
            hipError_t e = hipStreamWaitEvent(p.st->stream, p.marked, 0);
            p.marked = nullptr;
            return e;
        }
        hipError_t join() {
            if (!used) return hipSuccess;
            hipError_t e = hipEventRecord(st->join_ev, st->side);
            if (e == hipSuccess) e = hipStreamWaitEvent(st->stream, st->join_ev, 0);
            return e;
        }
    } pipe{st, {}, c.loss};
    MetaArgs &m = pipe.m;
    m.Z = st->at<float>(l.off_Z); m.zl = zl; m.y = rd->y; m.y_run_stride = yrs;
    m.L = st->at<double>(l.off_L); m.regret = st->at<double>(l.off_regret);
    m.last = l.off_last ? st->at<double>(l.off_last) : nullptr;
    m.eps = c.eps; m.K = (int)c.K; m.R = (int)c.R; m.n = (int)n;
    const PieceHook hook{&MetaPipe::piece, &pipe, &MetaPipe::beside, &MetaPipe::mark, &MetaPipe::wait_mark};
    const bool overlap = st->side != nullptr && st->tune.get(OCO_OPT_META_BESIDE) != 0;

    if (sparse) {
        SparseArgs a{};
        a.col = rd->col; a.val = rd->val; a.y = rd->y; a.y_run_stride = yrs;
        a.u = st->u_dev; a.seg_start = st->at<int64_t>(l.off_seg); a.S = (int)st->S;
        a.V = st->at<float>(l.off_V); a.sigma = st->at<double>(l.off_sigma); a.n2 = st->at<double>(l.off_n2);
        a.eta = st->at<float>(l.off_eta); a.Z = st->at<float>(l.off_Z); a.zl = zl;
        a.d = (int)c.d; a.K = (int)c.K; a.R = (int)c.R; a.nnz = c.sparse_nnz; a.RKp = l.RKp;
        a.t0 = t0; a.n = (int)n; a.D = c.D;
        a.scratch = st->at<char>(l.off_gram);
        a.optimistic = c.optimistic;
        if (c.optimistic) {
            a.ha = st->at<float>(l.off_ha); a.hp = st->at<float>(l.off_hp); a.hx = st->at<float>(l.off_x2last);
            a.last_col = st->at<int32_t>(l.off_lastcol); a.last_val = st->at<float>(l.off_lastval);
            a.xlast_dense = st->at<float>(l.off_xlast);
        }
        a.tune = &st->tune; a.clock = st->timing ? &st->clock : nullptr;
        e = launch_sparse_rounds(a, c.loss, st->stream, overlap ? &hook : nullptr);
    } else {
        DenseArgs a{};
        a.x = rd->x; a.x_run_stride = xrs; a.y = rd->y; a.y_run_stride = yrs;
        a.u = st->u_dev; a.seg_start = st->at<int64_t>(l.off_seg); a.S = (int)st->S;
        a.V = st->at<float>(l.off_V); a.sigma = st->at<float>(l.off_sigma);
        a.n2 = st->at<double>(l.off_n2); a.x2 = st->at<float>(l.off_X2);
        a.x2_run_stride = (int64_t)align_up((size_t)l.n_max, 64);
        a.eta = st->at<float>(l.off_eta); a.Z = st->at<float>(l.off_Z); a.zl = zl;
        a.d = (int)c.d; a.K = (int)c.K; a.R = (int)c.R; a.t0 = t0; a.n = (int)n; a.D = (float)c.D;
        a.x_shared = c.x_shared;
        a.vec_ok = (c.d % 4 == 0) && !mis(rd->x, 16) && (c.x_shared || xrs % 4 == 0);
        a.optimistic = c.optimistic;
        if (c.optimistic) {
            a.ha = st->at<float>(l.off_ha); a.hp = st->at<float>(l.off_hp);
            a.g01 = st->at<float>(l.off_G01);
            a.xlast = st->at<float>(l.off_xlast); a.x2last = st->at<float>(l.off_x2last);
        }
        a.tune = &st->tune; a.plan = &st->dense_plan; a.clock = st->timing ? &st->clock : nullptr;
        a.gram = l.off_gram ? st->at<float>(l.off_gram) : nullptr;
        a.n_max = l.n_max;
        e = launch_dense_rounds(a, c.loss, st->stream, overlap ? &hook : nullptr);
    }
    if (e != hipSuccess) return fail();
    // timing: [ev0, ev1] spans the round kernels, [ev1, ev2] whatever meta work is left after them
    if (st->timing && hipEventRecord(st->ev[1], st->stream) != hipSuccess) return fail();
    if (pipe.used) {
        if (pipe.join() != hipSuccess) return fail();
    } else if (launch_meta(m, c.loss, st->stream) != hipSuccess) {
        return fail();
    }
    if (st->timing) {
        if (hipEventRecord(st->ev[2], st->stream) != hipSuccess) return fail();
        st->timed = true;
    }
    st->t_done = t0 + n;
    return OCO_OK;
}

int oco_regret(oco_state *st, double *out_host)
{
    if (!st || !out_host) return OCO_EINVAL;
    if (st->failed) return OCO_EHIP;
    if (hipMemcpyAsync(out_host, st->at<double>(st->lay.off_regret), sizeof(double) * st->cfg.R,
                       hipMemcpyDeviceToHost, st->stream) != hipSuccess)
        return OCO_EHIP;
    return hipStreamSynchronize(st->stream) == hipSuccess ? OCO_OK : OCO_EHIP;
}

int oco_accel_bounds(oco_state *st, int64_t k, double alpha, double *out_dev)
{
    if (!st || !out_dev || k < 1 || !std::isfinite(alpha) || alpha < 0.0) return OCO_EINVAL;
    if (reinterpret_cast<uintptr_t>(out_dev) & 7u) return OCO_EINVAL;
    if (st->failed) return OCO_EHIP;
    if (st->t_done <= 0) return OCO_ESEQ;
    return launch_accel_bounds(st->at<double>(st->lay.off_regret), (int)st->cfg.R, st->t_done, k, alpha,
                               out_dev, st->stream) == hipSuccess ? OCO_OK : OCO_EHIP;
}

int oco_cum_losses(oco_state *st, double *out_host)
{
    if (!st || !out_host) return OCO_EINVAL;
    if (st->failed) return OCO_EHIP;
    if (hipMemcpyAsync(out_host, st->at<double>(st->lay.off_L), sizeof(double) * st->cfg.R * st->cfg.K,
                       hipMemcpyDeviceToHost, st->stream) != hipSuccess)
        return OCO_EHIP;
    return hipStreamSynchronize(st->stream) == hipSuccess ? OCO_OK : OCO_EHIP;
}

int oco_get_state(oco_state *st, float *W_dev, float *p_dev, float *wbar_dev)
{
    if (!st) return OCO_EINVAL;
    if (st->failed) return OCO_EHIP;
    auto mis = [](const void *p) { return (reinterpret_cast<uintptr_t>(p) & 3u) != 0; };
    if (mis(W_dev) || mis(p_dev) || mis(wbar_dev)) return OCO_EINVAL;
    ExportArgs a{};
    a.V = st->at<float>(st->lay.off_V);
    a.sigma = st->at<void>(st->lay.off_sigma);
    a.L = st->at<double>(st->lay.off_L);
    a.last = st->lay.off_last ? st->at<double>(st->lay.off_last) : nullptr;
    a.eps = st->cfg.eps;
    a.W = W_dev; a.p = p_dev; a.wbar = wbar_dev;
    a.d = (int)st->cfg.d; a.K = (int)st->cfg.K; a.R = (int)st->cfg.R; a.RKp = st->lay.RKp;
    a.sparse = st->cfg.sparse_nnz > 0;
    a.optimistic = st->cfg.optimistic;
    if (a.optimistic) {
        a.ha = st->at<float>(st->lay.off_ha); a.hp = st->at<float>(st->lay.off_hp);
        a.xlast = st->at<float>(st->lay.off_xlast); a.x2last = st->at<float>(st->lay.off_x2last);
        a.n2 = st->at<double>(st->lay.off_n2);
        a.x_shared = st->cfg.x_shared; a.D = (float)st->cfg.D;
    }
    return launch_export(a, st->stream) == hipSuccess ? OCO_OK : OCO_EHIP;
}

int oco_set_timing(oco_state *st, int enable)
{
    if (!st) return OCO_EINVAL;
    if (enable && st->is_static) return OCO_EUNSUPPORTED;     // would create events
    if (enable)
    {
        for (auto &e : st->ev)
            if (!e && hipEventCreate(&e) != hipSuccess) return OCO_EHIP;
        for (auto &e : st->clock.ev)
            if (!e && hipEventCreate(&e) != hipSuccess) return OCO_EHIP;
    }
    st->timing = enable != 0;
    st->timed = false;
    return OCO_OK;
}

int oco_last_timing(oco_state *st, float *ms_host)
{
    if (!st || !ms_host || !st->timing || !st->timed) return OCO_EINVAL;
    if (hipEventSynchronize(st->ev[2]) != hipSuccess) return OCO_EHIP;
    if (hipEventElapsedTime(&ms_host[0], st->ev[0], st->ev[1]) != hipSuccess) return OCO_EHIP;
    if (hipEventElapsedTime(&ms_host[1], st->ev[1], st->ev[2]) != hipSuccess) return OCO_EHIP;
    return OCO_OK;
}

int oco_last_kernel_timing(oco_state *st, float *ms_sum_host, int *timed_host, int *launches_host, const char **kernel)
{
    if (!st || !ms_sum_host || !timed_host || !launches_host || !st->timing || !st->timed) return OCO_EINVAL;
    if (hipEventSynchronize(st->ev[2]) != hipSuccess) return OCO_EHIP;
    float sum = 0.f;
    for (int i = 0; i < st->clock.timed; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, st->clock.ev[2 * i], st->clock.ev[2 * i + 1]) != hipSuccess) return OCO_EHIP;
        sum += ms;
    }
    *ms_sum_host = sum;
    *timed_host = st->clock.timed;
    *launches_host = st->clock.launches;
    if (kernel) *kernel = st->clock.kernel;
    return OCO_OK;
}

int64_t oco_rounds_done(const oco_state *st) { return st ? st->t_done : (int64_t)OCO_EINVAL; }

void oco_destroy(oco_state *st) { delete st; }

const char *oco_strerror(int status)
{
    switch (status) {
        case OCO_OK: return "ok";
        case OCO_EINVAL: return "invalid argument";
        case OCO_ESEQ: return "t0 does not continue the rounds already consumed";
        case OCO_ERANGE: return "round range or segment count out of range";
        case OCO_ENOMEM: return "workspace too small";
        case OCO_EHIP: return "HIP runtime error";
        case OCO_ENOCOMP: return "comparator not set";
        case OCO_EUNSUPPORTED: return "shape not supported by the kernels";
        default: return "unknown status";
    }
}

}  // extern "C"
