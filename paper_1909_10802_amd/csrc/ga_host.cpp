// Host side of libga: the C ABI of include/ga.h, the integer bookkeeping of
// the master (step counter, iter[], delays: Alg. 3 / Alg. 5), the per-arrival
// scalars (step size, Alg. 14 bias correction) and the arrival-schedule
// simulator.  Device work is delegated to the launchers in the .hip files.

#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "ga_internal.h"

struct ga_ctx {
    uint64_t N = 0;
    uint32_t W = 0;
    int family = GA_FAMILY_MOMENTUM;
    int mode = GA_MODE_GA;
    float eta_max = 0.f, lr = 0.f, gamma = 0.f, beta = 0.999f, eps = 1e-8f;
    float beta1 = 0.9f, beta2 = 0.999f, adam_eps = 1e-8f;
    bool track_gap = false;
    bool nesterov = false;
    hipStream_t stream = nullptr;
    ga::StatePtrs st{};
    ga_arrival* dev_table = nullptr;
    ga::AdamRow* dev_adam_table = nullptr;
    const void** dev_grad_table = nullptr;   // one gradient-buffer pointer per row of the arrival table
    size_t state_bytes = 0;        // theta .. last state row, contiguous in the workspace
    ga::DiagPartial* dev_partials = nullptr;
    uint64_t k = 0;
    std::vector<uint64_t> iter;
    // delays of the most recent arrivals: a ring of at most kDelayLog entries (a master that runs for
    // millions of steps must not grow), delay_next is the slot the next delay goes to
    std::vector<uint64_t> delays;
    uint64_t delay_next = 0;
    // pinned staging for one chunk of the arrival table (and Adam's rows); `staged` is recorded after
    // the upload so that the next chunk does not overwrite rows that are still being copied
    ga_arrival* rows = nullptr;
    ga::AdamRow* adam_rows = nullptr;
    const void** grad_rows = nullptr;
    hipEvent_t staged = nullptr;
    bool staged_pending = false;
    int gap_scope = GA_GAP_PARAMETER;
    // layer-wise / global Gap: the chunk sums on the device are those of the next arrival of this worker
    // (valid only between two arrivals of one ga_run_schedule call)
    bool layer_sums_ready = false;
    uint32_t layer_sums_worker = 0;
    ga::LayerTables layers{};
    std::vector<ga::LayerChunk> host_chunks;   // uploaded at create; kept for the lifetime of the context
    std::vector<ga::LayerSpan> host_spans;
    std::string err;
};

namespace {

thread_local std::string g_create_error;

int fail(ga_ctx* ctx, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (ctx) ctx->err = buf; else g_create_error = buf;
    return code;
}

void record_delay(ga_ctx* ctx, uint64_t tau) {
    if (ctx->delays.size() < ga::kDelayLog) {
        ctx->delays.push_back(tau);
    } else {
        ctx->delays[ctx->delay_next] = tau;
        ctx->delay_next = (ctx->delay_next + 1) % ga::kDelayLog;
    }
}

int hip_fail(ga_ctx* ctx, hipError_t e, const char* what) {
    return fail(ctx, GA_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

bool is_gap_mode(int mode) { return mode == GA_MODE_GA || mode == GA_MODE_GA_HINGE; }
bool valid_mode(int mode) { return mode >= GA_MODE_ASGD && mode <= GA_MODE_GA_HINGE; }

uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

struct Layout {
    uint64_t Np, n_rows;
    size_t off_theta, off_v, off_m, off_snaps, off_worker_v, off_v2, off_table, off_partials, total;
    size_t worker_bytes;   // bytes between consecutive workers' regions
    size_t off_chunks, off_spans, off_layer_partials, off_gaps, off_adam_table, off_grad_table;
};

// Chunks of at most kLayerChunk parameters, never across a layer boundary.  sizes == nullptr: one layer of N.
bool build_layer_tables(uint64_t N, uint32_t n_layers, const uint64_t* sizes, std::vector<ga::LayerChunk>* chunks,
                        std::vector<ga::LayerSpan>* spans, uint64_t* n_chunks_out) {
    uint64_t start = 0, n_chunks = 0;
    for (uint32_t p = 0; p < n_layers; ++p) {
        const uint64_t len = sizes ? sizes[p] : N;
        if (len == 0 || len > N - start) return false;
        // cuts inside a layer fall on 256-byte boundaries of the arrays, so only the first and the last
        // chunk of a layer have an unaligned edge
        const uint64_t base = start & ~(uint64_t)63, end = start + len;
        const uint64_t c = (end - base + ga::kLayerChunk - 1) / ga::kLayerChunk;
        if (spans) spans->push_back(ga::LayerSpan{(uint32_t)n_chunks, (uint32_t)c});
        if (chunks)
            for (uint64_t i = 0; i < c; ++i) {
                const uint64_t lo = i == 0 ? start : base + i * ga::kLayerChunk;
                const uint64_t hi = base + (i + 1) * ga::kLayerChunk < end ? base + (i + 1) * ga::kLayerChunk : end;
                chunks->push_back(ga::LayerChunk{lo, (uint32_t)(hi - lo), p});
            }
        n_chunks += c;
        start += len;
    }
    *n_chunks_out = n_chunks;
    return start == N && n_chunks < 0x7FFFFFFFull;
}

// theta, v, m [ADAM: and v2] interleaved by tiles (ga_internal.h) | W snapshot rows [DANA: W tiled pairs of snapshot
// and worker momentum] | arrival, Adam and gradient-pointer tables | reduction partials
Layout layout_for(uint64_t N, uint32_t W, int family, uint64_t n_chunks = 0, uint32_t n_layers = 0) {
    Layout L;
    L.Np = round_up(N, 64);                  // every row starts 256-byte aligned
    const size_t row = (size_t)L.Np * sizeof(float);
    const size_t tile = (size_t)ga::kStateTile * sizeof(float);
    L.off_theta = 0;
    L.off_v = tile;
    L.off_m = 2 * tile;
    L.off_v2 = family == GA_FAMILY_ADAM ? 3 * tile : 0;      // ADAM: the fourth tiled array
    const size_t tiled_row = (size_t)round_up(N, ga::kStateTile) * sizeof(float);
    L.off_snaps = (size_t)ga::state_rows(family) * tiled_row;
    L.n_rows = (uint64_t)W;                  // per-worker regions after the tiled state
    L.off_worker_v = 0;
    L.worker_bytes = row;                    // a snapshot row
    if (family == GA_FAMILY_DANA) {          // snapshot and v_i of a worker: a tiled pair (ga_internal.h)
        L.worker_bytes = 2 * tiled_row;
        L.off_worker_v = L.off_snaps + tile;
    }
    L.off_table = L.off_snaps + L.n_rows * L.worker_bytes;
    L.off_adam_table = L.off_table + round_up((uint64_t)ga::kTableCap * sizeof(ga_arrival), 256);
    L.off_grad_table = L.off_adam_table + round_up((uint64_t)ga::kTableCap * sizeof(ga::AdamRow), 256);
    L.off_partials = L.off_grad_table + round_up((uint64_t)ga::kTableCap * sizeof(void*), 256);
    L.total = L.off_partials + round_up((uint64_t)(ga::kDiagMaxBlocks + 1) * sizeof(ga::DiagPartial), 256);
    L.off_chunks = L.total;
    L.off_spans = L.off_chunks + round_up(n_chunks * sizeof(ga::LayerChunk), 256);
    L.off_layer_partials = L.off_spans + round_up((uint64_t)n_layers * sizeof(ga::LayerSpan), 256);
    L.off_gaps = L.off_layer_partials + round_up(n_chunks * sizeof(ga::LayerPartial), 256);
    L.total = L.off_gaps + round_up((uint64_t)n_layers * sizeof(float), 256);
    return L;
}

// (float)(1 / (1 - beta^k)) with the power, difference and quotient in double; 0 for k = 0
// (Alg. 14: m_0 = 0, so m-hat_0 is taken as 0).
float inverse_bias_correction(float beta, uint64_t k) {
    if (k == 0) return 0.0f;
    return (float)(1.0 / (1.0 - std::pow((double)beta, (double)k)));
}

// ----------------------------------------------------------- schedule draws
// Philox4x32-10 (Salmon et al., SC'11), host copy used for iteration times.
struct Block4 { uint32_t w[4]; };

Block4 philox_block(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint64_t key) {
    uint32_t k0 = (uint32_t)key, k1 = (uint32_t)(key >> 32);
    for (int r = 0; r < 10; ++r) {
        const uint64_t a = 0xD2511F53ull * c0;
        const uint64_t b = 0xCD9E8D57ull * c2;
        const uint32_t t0 = (uint32_t)(b >> 32) ^ c1 ^ k0;
        const uint32_t t2 = (uint32_t)(a >> 32) ^ c3 ^ k1;
        c1 = (uint32_t)b;
        c3 = (uint32_t)a;
        c0 = t0;
        c2 = t2;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return Block4{{c0, c1, c2, c3}};
}

double unit53(uint32_t lo, uint32_t hi) {   // 53 random bits -> [0, 1)
    return (double)((((uint64_t)hi << 32) | lo) >> 11) * 0x1.0p-53;
}

double normal_of(const Block4& b) {          // Box-Muller, double
    const double radius = std::sqrt(-2.0 * std::log1p(-unit53(b.w[0], b.w[1])));
    return radius * std::cos(6.283185307179586476925286766559 * unit53(b.w[2], b.w[3]));
}

constexpr uint32_t kTagTime = 0x54494D45u;   // counter word 3: per-iteration draw
constexpr uint32_t kTagMean = 0x4D45414Eu;   // counter word 3: per-worker draw

constexpr uint32_t kTagGamma = 0x47000000u;  // counter word 3 of a gamma draw: + 65536 * kind + attempt

// Gamma variate, shape >= 1 (Marsaglia & Tsang, ACM TOMS 26, 2000): squeeze-free form with one
// normal and one uniform per attempt, both taken from the Philox block of that attempt.
double gamma_variate(double shape, double scale, uint64_t seed, uint32_t c0, uint32_t c1, uint32_t c2, uint32_t kind) {
    const double d = shape - 1.0 / 3.0;
    const double c = 1.0 / std::sqrt(9.0 * d);
    for (uint32_t attempt = 0; attempt < 65536; ++attempt) {
        const Block4 b = philox_block(c0, c1, c2, kTagGamma + 65536u * kind + attempt, seed);
        const double radius = std::sqrt(-2.0 * std::log1p(-unit53(b.w[0], b.w[1])));
        const double z = radius * std::cos(6.283185307179586476925286766559 * (((double)b.w[2] + 0.5) / 4294967296.0));
        const double accept = ((double)b.w[3] + 0.5) / 4294967296.0;
        double v = 1.0 + c * z;
        if (v <= 0.0) continue;
        v = v * v * v;
        if (std::log(accept) < 0.5 * z * z + d - d * v + d * std::log(v)) return d * v * scale;
    }
    return std::nan("");
}

class TimeModel {
  public:
    TimeModel(const ga_time_model& m, uint64_t seed, uint32_t W) : m_(m), seed_(seed) {
        if (m.dist == GA_DIST_HETERO) {
            mean_.resize(W);
            for (uint32_t w = 0; w < W; ++w) mean_[w] = std::exp(m.sigma * normal_of(philox_block(w, 0, 0, kTagMean, seed)));
        } else if (m.dist == GA_DIST_GAMMA_HOMO) {          // Alg. 12: one q for the whole run
            a_task_ = 1.0 / (m.v_task * m.v_task);
            a_mach_ = 1.0 / (m.v_mach * m.v_mach);
            mean_.assign(1, gamma_variate(a_task_, m.mean / a_task_, seed, 0, 0, 0, 1));
        } else if (m.dist == GA_DIST_GAMMA_HETERO) {        // Alg. 13: one p per machine
            a_task_ = 1.0 / (m.v_task * m.v_task);
            a_mach_ = 1.0 / (m.v_mach * m.v_mach);
            mean_.resize(W);
            for (uint32_t w = 0; w < W; ++w) mean_[w] = gamma_variate(a_mach_, m.mean / a_mach_, seed, w, 0, 0, 2);
        }
    }
    double draw(uint32_t w, uint64_t n) const {
        if (m_.dist == GA_DIST_GAMMA_HOMO)
            return gamma_variate(a_mach_, mean_[0] / a_mach_, seed_, (uint32_t)n, (uint32_t)(n >> 32), w, 0);
        if (m_.dist == GA_DIST_GAMMA_HETERO)
            return gamma_variate(a_task_, mean_[w] / a_task_, seed_, (uint32_t)n, (uint32_t)(n >> 32), w, 0);
        const Block4 b = philox_block((uint32_t)n, (uint32_t)(n >> 32), w, kTagTime, seed_);
        if (m_.dist == GA_DIST_LOGNORMAL) return std::exp(m_.sigma * normal_of(b));
        const double e = -std::log1p(-unit53(b.w[0], b.w[1]));
        return m_.dist == GA_DIST_HETERO ? mean_[w] * e : e;
    }

  private:
    ga_time_model m_;
    uint64_t seed_;
    double a_task_ = 0.0, a_mach_ = 0.0;
    std::vector<double> mean_;
};

int check_time_model(const ga_time_model* m) {
    if (!m) return fail(nullptr, GA_ERR_ARG, "time model is null");
    if (m->dist < GA_DIST_EXP || m->dist > GA_DIST_GAMMA_HETERO) return fail(nullptr, GA_ERR_ARG, "unknown time distribution %d", m->dist);
    if ((m->dist == GA_DIST_LOGNORMAL || m->dist == GA_DIST_HETERO) && !(m->sigma >= 0.0 && std::isfinite(m->sigma)))
        return fail(nullptr, GA_ERR_ARG, "time model: sigma must be finite and >= 0");
    if (m->dist == GA_DIST_GAMMA_HOMO || m->dist == GA_DIST_GAMMA_HETERO) {
        if (!(m->mean > 0.0) || !std::isfinite(m->mean)) return fail(nullptr, GA_ERR_ARG, "time model: mean must be finite and > 0");
        if (!(m->v_mach > 0.0 && m->v_mach <= 1.0) || !(m->v_task > 0.0 && m->v_task <= 1.0))
            return fail(nullptr, GA_ERR_ARG, "time model: v_mach and v_task must be in (0, 1]");
    }
    return GA_OK;
}

// FIFO service of the workers' finish times; ties to the lowest id.  Calls visit(arrival, worker, time).
template <typename Visit>
void replay_arrivals(const TimeModel& model, uint32_t W, uint64_t T, Visit visit) {
    std::vector<double> finish(W);
    std::vector<uint64_t> done(W, 0);
    for (uint32_t w = 0; w < W; ++w) finish[w] = model.draw(w, 0);
    for (uint64_t a = 0; a < T; ++a) {
        uint32_t first = 0;                     // earliest finish; strict '<' keeps the lowest id on ties
        for (uint32_t w = 1; w < W; ++w)
            if (finish[w] < finish[first]) first = w;
        visit(a, first, finish[first]);
        done[first] += 1;
        finish[first] = finish[first] + model.draw(first, done[first]);
    }
}

// ----------------------------------------------------------- per-arrival scalars
ga_arrival make_row(uint32_t worker, uint64_t k, uint64_t tau, int mode, float eta_k, float beta) {
    ga_arrival r;
    r.worker = worker;
    r.tau = (float)tau;
    r.lr = (mode == GA_MODE_SA_STEP) ? eta_k / r.tau : eta_k;
    r.inv_bc_prev = inverse_bias_correction(beta, k - 1);
    return r;
}

// Rows (and integer delays) of T arrivals after step k0.  Arguments are already validated.
void plan(uint64_t T, const uint32_t* schedule, uint64_t k0, uint64_t* iter, int mode, float eta_k, float beta,
          ga_arrival* rows, uint64_t* taus, const float* eta_table = nullptr) {
    for (uint64_t a = 0; a < T; ++a) {
        const uint64_t k = k0 + a + 1;
        const uint32_t w = schedule[a];
        const uint64_t tau = k - iter[w];
        rows[a] = make_row(w, k, tau, mode, eta_table ? eta_table[a] : eta_k, beta);
        if (taus) taus[a] = tau;
        iter[w] = k;
    }
}

ga::StepConst step_const(const ga_ctx* c, const ga_arrival& r, uint64_t k) {
    ga::StepConst s = {};
    s.gamma = c->gamma;
    s.lr = r.lr;
    s.tau = r.tau;
    s.inv_bc_prev = r.inv_bc_prev;
    s.eta_max = c->eta_max;
    s.eps = c->eps;
    s.beta = c->beta;
    s.one_minus_beta = 1.0f - c->beta;
    s.eta_gamma = r.lr * c->gamma;
    if (c->family == GA_FAMILY_ADAM) {
        s.beta1 = c->beta1;
        s.omb1 = 1.0f - c->beta1;
        s.beta2 = c->beta2;
        s.omb2 = 1.0f - c->beta2;
        s.adam_eps = c->adam_eps;
        s.inv_bc1 = inverse_bias_correction(c->beta1, k);
        s.inv_bc2 = inverse_bias_correction(c->beta2, k);
    }
    return s;
}

ga::RunConst run_const(const ga_ctx* c, const ga_grad_source* src) {
    ga::RunConst r;
    r.gamma = c->gamma;
    r.eta_max = c->eta_max;
    r.eps = c->eps;
    r.beta = c->beta;
    r.one_minus_beta = 1.0f - c->beta;
    r.beta1 = c->beta1;
    r.omb1 = 1.0f - c->beta1;
    r.beta2 = c->beta2;
    r.omb2 = 1.0f - c->beta2;
    r.adam_eps = c->adam_eps;
    r.sigma = src->sigma;
    r.seed_lo = (uint32_t)src->seed;
    r.seed_hi = (uint32_t)(src->seed >> 32);
    return r;
}

bool keeps_m(const ga_ctx* c) { return is_gap_mode(c->mode) || c->track_gap; }

int check_quadratic_source(ga_ctx* ctx, const ga_grad_source* src) {
    if (!src->dev_a || !src->dev_theta_star) return fail(ctx, GA_ERR_ARG, "quadratic source: dev_a / dev_theta_star is null");
    if (((uintptr_t)src->dev_a & 15u) || ((uintptr_t)src->dev_theta_star & 15u))
        return fail(ctx, GA_ERR_ALIGN, "quadratic source: dev_a / dev_theta_star must be 16-byte aligned");
    if (!std::isfinite(src->sigma)) return fail(ctx, GA_ERR_ARG, "quadratic source: sigma is not finite");
    return GA_OK;
}

// One arrival through the fused kernel; the bookkeeping is committed only if the launch succeeded.
// next_worker (layer-wise and global Gap only): the worker of the arrival that follows in the same
// schedule, or -1; the update pass then prepares that arrival's norms (see launch_apply_layerwise).
int apply_one(ga_ctx* ctx, uint32_t worker, const void* dev_grad, int dtype, bool write_snap, float eta_k,
              int64_t next_worker = -1) {
    const uint64_t k = ctx->k + 1;
    const uint64_t tau = k - ctx->iter[worker];
    const ga_arrival row = make_row(worker, k, tau, ctx->mode, eta_k, ctx->beta);
    const ga::StepConst sc = step_const(ctx, row, k);
    hipError_t e;
    if (ctx->gap_scope != GA_GAP_PARAMETER) {
        const bool ready = ctx->layer_sums_ready && ctx->layer_sums_worker == worker;
        ctx->layer_sums_ready = false;
        e = ga::launch_apply_layerwise(ctx->st, ctx->N, worker, dev_grad, dtype, ctx->mode, ctx->nesterov, ctx->layers, sc,
                                       ready, next_worker, ctx->stream);
        if (e == hipSuccess && next_worker >= 0) {
            ctx->layer_sums_ready = true;
            ctx->layer_sums_worker = (uint32_t)next_worker;
        }
    } else if (ctx->family == GA_FAMILY_DANA)
        e = ga::launch_apply_dana(ctx->st, ctx->N, worker, dev_grad, dtype, ctx->mode, keeps_m(ctx), write_snap, sc, ctx->stream);
    else if (ctx->family == GA_FAMILY_ADAM)
        e = ga::launch_apply_adam(ctx->st, ctx->N, worker, dev_grad, dtype, ctx->mode, keeps_m(ctx), write_snap, sc, ctx->stream);
    else
        e = ga::launch_apply(ctx->st, ctx->N, worker, dev_grad, dtype, ctx->mode, ctx->nesterov, keeps_m(ctx), write_snap, sc, ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "apply launch");
    ctx->k = k;
    ctx->iter[worker] = k;
    record_delay(ctx, tau);
    return GA_OK;
}

// theta, v, m (v2) and, in the DANA master, the per-worker arrays are tiled in the workspace (ga_internal.h): a kernel
// gathers / scatters them; plain rows are copied.
// Arrays per tile at p: theta, v, m (v2) are tiled with the state, a DANA worker's snapshot and v_i as a pair; 1: a row.
int tiled_rows(const ga_ctx* ctx, const float* p) {
    if (p == ctx->st.theta || p == ctx->st.v || p == ctx->st.m || (ctx->st.v2 && p == ctx->st.v2)) return ctx->st.rows;
    return ctx->st.snap_rows;   // every other array handed to the copy helpers is a per-worker one
}

int copy_out(ga_ctx* ctx, float* dst, const float* src) {
    if (!ctx) return GA_ERR_ARG;
    if (!dst) return fail(ctx, GA_ERR_ARG, "destination is null");
    const int rows = tiled_rows(ctx, src);
    const hipError_t e = rows > 1
                             ? ga::launch_state_get(src, rows, dst, ctx->N, ctx->stream)
                             : hipMemcpyAsync(dst, src, ctx->N * sizeof(float), hipMemcpyDeviceToDevice, ctx->stream);
    return e == hipSuccess ? GA_OK : hip_fail(ctx, e, "copy");
}

int copy_in(ga_ctx* ctx, float* dst, const float* src) {
    if (!ctx) return GA_ERR_ARG;
    if (!src) return fail(ctx, GA_ERR_ARG, "source is null");
    const int rows = tiled_rows(ctx, dst);
    const hipError_t e = rows > 1
                             ? ga::launch_state_put(dst, rows, src, ctx->N, ctx->stream)
                             : hipMemcpyAsync(dst, src, ctx->N * sizeof(float), hipMemcpyDeviceToDevice, ctx->stream);
    return e == hipSuccess ? GA_OK : hip_fail(ctx, e, "copy");
}

}  // namespace

extern "C" {

const char* ga_version(void) { return "0.1"; }

const char* ga_last_error(const ga_ctx* ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

// ------------------------------------------------------------------ host only
int ga_simulate_schedule_ex(uint32_t n_workers, uint64_t T, const ga_time_model* model, uint64_t seed,
                            uint32_t* host_schedule, double* host_finish_times) {
    if (n_workers == 0 || (T > 0 && !host_schedule)) return fail(nullptr, GA_ERR_ARG, "simulate_schedule: bad argument");
    const int rc = check_time_model(model);
    if (rc != GA_OK) return rc;
    const TimeModel tm(*model, seed, n_workers);
    replay_arrivals(tm, n_workers, T, [&](uint64_t a, uint32_t w, double t) {
        host_schedule[a] = w;
        if (host_finish_times) host_finish_times[a] = t;
    });
    return GA_OK;
}

int ga_simulate_schedule(uint32_t n_workers, uint64_t T, int dist, double sigma, uint64_t seed,
                         uint32_t* host_schedule) {
    if (dist < GA_DIST_EXP || dist > GA_DIST_HETERO) return fail(nullptr, GA_ERR_ARG, "simulate_schedule: unknown distribution");
    const ga_time_model m = {dist, sigma, 0.0, 0.0, 0.0};
    return ga_simulate_schedule_ex(n_workers, T, &m, seed, host_schedule, nullptr);
}

int ga_simulate_speedup(uint32_t n_workers, uint64_t iters, const ga_time_model* model, uint64_t seed,
                        double* asgd_wall, double* ssgd_wall) {
    if (n_workers == 0 || !asgd_wall || !ssgd_wall) return fail(nullptr, GA_ERR_ARG, "simulate_speedup: bad argument");
    const int rc = check_time_model(model);
    if (rc != GA_OK) return rc;
    const TimeModel tm(*model, seed, n_workers);
    double sync = 0.0;
    for (uint64_t i = 0; i < iters; ++i) {          // SSGD: a barrier after every batch
        double slowest = 0.0;
        for (uint32_t w = 0; w < n_workers; ++w) {
            const double t = tm.draw(w, i);
            if (t > slowest) slowest = t;
        }
        sync += slowest;
    }
    double last = 0.0;
    replay_arrivals(tm, n_workers, (uint64_t)n_workers * iters, [&](uint64_t, uint32_t, double t) { last = t; });
    *asgd_wall = last;
    *ssgd_wall = sync;
    return GA_OK;
}

int ga_warmup_lr(float eta, uint32_t n_workers, uint64_t warmup_steps, uint64_t k0, uint64_t T, float* host_eta) {
    if (!(eta > 0.f) || !std::isfinite(eta) || n_workers == 0 || (T > 0 && !host_eta))
        return fail(nullptr, GA_ERR_ARG, "warmup_lr: bad argument");
    const double lo = (double)eta / (double)n_workers;
    for (uint64_t a = 0; a < T; ++a) {
        const uint64_t k = k0 + a + 1;
        double x = (double)eta;
        if (k < warmup_steps) x = lo + ((double)eta - lo) * ((double)k / (double)warmup_steps);
        host_eta[a] = (float)x;
    }
    return GA_OK;
}

int ga_delays_from_schedule(uint32_t n_workers, uint64_t T, const uint32_t* host_schedule, uint64_t k0,
                            uint64_t* host_iter, uint64_t* host_tau) {
    if (n_workers == 0 || !host_iter || (T > 0 && (!host_schedule || !host_tau)))
        return fail(nullptr, GA_ERR_ARG, "delays_from_schedule: bad argument");
    for (uint64_t a = 0; a < T; ++a)
        if (host_schedule[a] >= n_workers) return fail(nullptr, GA_ERR_WORKER, "schedule[%llu] = %u >= n_workers", (unsigned long long)a, host_schedule[a]);
    for (uint32_t w = 0; w < n_workers; ++w)
        if (host_iter[w] > k0) return fail(nullptr, GA_ERR_ARG, "iter[%u] is ahead of k0", w);
    for (uint64_t a = 0; a < T; ++a) {
        const uint64_t k = k0 + a + 1;
        uint64_t& last = host_iter[host_schedule[a]];
        host_tau[a] = k - last;
        last = k;
    }
    return GA_OK;
}

int ga_plan_arrivals(uint32_t n_workers, uint64_t T, const uint32_t* host_schedule, uint64_t k0, uint64_t* host_iter,
                     int mode, float eta_k, float beta, ga_arrival* host_rows) {
    if (n_workers == 0 || !host_iter || (T > 0 && (!host_schedule || !host_rows)) || !valid_mode(mode))
        return fail(nullptr, GA_ERR_ARG, "plan_arrivals: bad argument");
    if (!(eta_k > 0.f) || !std::isfinite(eta_k) || !(beta >= 0.f && beta < 1.f))
        return fail(nullptr, GA_ERR_ARG, "plan_arrivals: eta_k must be > 0 and beta in [0,1)");
    for (uint64_t a = 0; a < T; ++a)
        if (host_schedule[a] >= n_workers) return fail(nullptr, GA_ERR_WORKER, "schedule[%llu] = %u >= n_workers", (unsigned long long)a, host_schedule[a]);
    for (uint32_t w = 0; w < n_workers; ++w)
        if (host_iter[w] > k0) return fail(nullptr, GA_ERR_ARG, "iter[%u] is ahead of k0", w);
    plan(T, host_schedule, k0, host_iter, mode, eta_k, beta, host_rows, nullptr);
    return GA_OK;
}

// ------------------------------------------------------------------ context
void ga_config_init(ga_config* cfg) {
    if (!cfg) return;
    cfg->N = 0;
    cfg->n_workers = 0;
    cfg->family = GA_FAMILY_MOMENTUM;
    cfg->mode = GA_MODE_GA;
    cfg->eta = 0.1f;
    cfg->gamma = 0.9f;
    cfg->beta = 0.999f;
    cfg->eps = 1e-8f;
    cfg->adam_beta1 = 0.9f;
    cfg->adam_beta2 = 0.999f;
    cfg->adam_eps = 1e-8f;
    cfg->track_gap = 0;
    cfg->gap_scope = GA_GAP_PARAMETER;
    cfg->n_layers = 0;
    cfg->host_layer_sizes = nullptr;
    cfg->nesterov = 0;
}

// Number of layers and chunks a configuration asks for; false if the layer description is invalid.
static bool layer_counts(const ga_config* cfg, uint32_t* n_layers, uint64_t* n_chunks) {
    *n_layers = 0;
    *n_chunks = 0;
    if (cfg->gap_scope == GA_GAP_PARAMETER) return true;
    if (cfg->gap_scope == GA_GAP_GLOBAL) {
        *n_layers = 1;
        return build_layer_tables(cfg->N, 1, nullptr, nullptr, nullptr, n_chunks);
    }
    if (cfg->gap_scope != GA_GAP_LAYER || cfg->n_layers == 0 || !cfg->host_layer_sizes) return false;
    *n_layers = cfg->n_layers;
    return build_layer_tables(cfg->N, cfg->n_layers, cfg->host_layer_sizes, nullptr, nullptr, n_chunks);
}

size_t ga_workspace_bytes_ex(const ga_config* cfg) {
    if (!cfg || cfg->N == 0 || cfg->n_workers == 0) return 0;
    if (cfg->family < GA_FAMILY_MOMENTUM || cfg->family > GA_FAMILY_ADAM) return 0;
    uint32_t n_layers;
    uint64_t n_chunks;
    if (!layer_counts(cfg, &n_layers, &n_chunks)) return 0;
    return layout_for(cfg->N, cfg->n_workers, cfg->family, n_chunks, n_layers).total;
}

size_t ga_workspace_bytes(uint64_t N, uint32_t n_workers) {
    if (N == 0 || n_workers == 0) return 0;
    return layout_for(N, n_workers, GA_FAMILY_MOMENTUM).total;
}

int ga_create_ex(ga_ctx** out, const ga_config* cfg, void* dev_workspace, size_t workspace_bytes, void* hip_stream) {
    if (!out) return fail(nullptr, GA_ERR_ARG, "create: out is null");
    *out = nullptr;
    if (!cfg) return fail(nullptr, GA_ERR_ARG, "create: configuration is null");
    const uint64_t N = cfg->N;
    const uint32_t n_workers = cfg->n_workers;
    if (N == 0 || n_workers == 0) return fail(nullptr, GA_ERR_ARG, "create: N and n_workers must be positive");
    if (N > (1ull << 40)) return fail(nullptr, GA_ERR_ARG, "create: N too large");
    if (cfg->family < GA_FAMILY_MOMENTUM || cfg->family > GA_FAMILY_ADAM) return fail(nullptr, GA_ERR_ARG, "create: unknown family %d", cfg->family);
    if (!(cfg->eta > 0.f) || !std::isfinite(cfg->eta)) return fail(nullptr, GA_ERR_ARG, "create: eta must be finite and > 0");
    if (!(std::fabs(cfg->gamma) < 1.f)) return fail(nullptr, GA_ERR_ARG, "create: |gamma| must be < 1");
    if (!valid_mode(cfg->mode)) return fail(nullptr, GA_ERR_ARG, "create: unknown mode %d", cfg->mode);
    if (cfg->mode == GA_MODE_SA_STEP && cfg->family != GA_FAMILY_MOMENTUM)
        return fail(nullptr, GA_ERR_ARG, "create: GA_MODE_SA_STEP exists for the momentum family only");
    if (cfg->nesterov && cfg->family != GA_FAMILY_MOMENTUM)
        return fail(nullptr, GA_ERR_ARG, "create: the Nesterov form exists for the momentum family only");
    if (!(cfg->beta >= 0.f && cfg->beta < 1.f)) return fail(nullptr, GA_ERR_ARG, "create: beta must be in [0,1)");
    if (!(cfg->eps > 0.f) || !std::isfinite(cfg->eps)) return fail(nullptr, GA_ERR_ARG, "create: eps must be finite and > 0");
    if (cfg->family == GA_FAMILY_ADAM) {
        if (!(cfg->adam_beta1 >= 0.f && cfg->adam_beta1 < 1.f) || !(cfg->adam_beta2 >= 0.f && cfg->adam_beta2 < 1.f))
            return fail(nullptr, GA_ERR_ARG, "create: Adam betas must be in [0,1)");
        if (!(cfg->adam_eps > 0.f) || !std::isfinite(cfg->adam_eps)) return fail(nullptr, GA_ERR_ARG, "create: adam_eps must be finite and > 0");
    }
    uint32_t n_layers;
    uint64_t n_chunks;
    if (!layer_counts(cfg, &n_layers, &n_chunks))
        return fail(nullptr, GA_ERR_ARG, "create: invalid gap scope or layer sizes (each > 0, summing to N)");
    if (cfg->gap_scope != GA_GAP_PARAMETER &&
        (cfg->family != GA_FAMILY_MOMENTUM || (cfg->mode != GA_MODE_GA && cfg->mode != GA_MODE_GA_HINGE)))
        return fail(nullptr, GA_ERR_ARG, "create: layer-wise / global Gap exists for the momentum family in the GA modes only");
    if (!dev_workspace) return fail(nullptr, GA_ERR_ARG, "create: workspace is null");
    const Layout L = layout_for(N, n_workers, cfg->family, n_chunks, n_layers);
    if (((uintptr_t)dev_workspace & 255u) != 0) return fail(nullptr, GA_ERR_ALIGN, "create: workspace must be 256-byte aligned");
    if (workspace_bytes < L.total)
        return fail(nullptr, GA_ERR_ALIGN, "create: workspace has %zu bytes, %zu needed", workspace_bytes, L.total);

    ga_ctx* c = new (std::nothrow) ga_ctx;
    if (!c) return fail(nullptr, GA_ERR_ARG, "create: out of host memory");
    c->N = N;
    c->W = n_workers;
    c->family = cfg->family;
    c->mode = cfg->mode;
    c->eta_max = c->lr = cfg->eta;
    c->gamma = cfg->family == GA_FAMILY_ADAM ? 0.0f : cfg->gamma;
    c->beta = cfg->beta;
    c->eps = cfg->eps;
    c->beta1 = cfg->adam_beta1;
    c->beta2 = cfg->adam_beta2;
    c->adam_eps = cfg->adam_eps;
    c->track_gap = cfg->track_gap != 0;
    c->nesterov = cfg->nesterov != 0;
    c->stream = static_cast<hipStream_t>(hip_stream);
    char* base = static_cast<char*>(dev_workspace);
    c->st.theta = reinterpret_cast<float*>(base + L.off_theta);
    c->st.v = reinterpret_cast<float*>(base + L.off_v);
    c->st.m = reinterpret_cast<float*>(base + L.off_m);
    c->st.snaps = reinterpret_cast<float*>(base + L.off_snaps);
    c->st.worker_v = L.off_worker_v ? reinterpret_cast<float*>(base + L.off_worker_v) : nullptr;
    c->st.v2 = L.off_v2 ? reinterpret_cast<float*>(base + L.off_v2) : nullptr;
    c->st.rows = ga::state_rows(cfg->family);
    c->st.snap_rows = ga::snapshot_rows(cfg->family);
    c->st.stride = L.worker_bytes / sizeof(float);
    c->st.resident_bytes = ga::kResidentBytes;
    c->dev_table = reinterpret_cast<ga_arrival*>(base + L.off_table);
    c->dev_adam_table = reinterpret_cast<ga::AdamRow*>(base + L.off_adam_table);
    c->dev_grad_table = reinterpret_cast<const void**>(base + L.off_grad_table);
    c->dev_partials = reinterpret_cast<ga::DiagPartial*>(base + L.off_partials);
    c->iter.assign(n_workers, 0);

    c->gap_scope = cfg->gap_scope;
    c->state_bytes = L.off_table;
    // the tiled arrays and all rows are contiguous: one fill
    hipError_t e = ga::launch_fill(c->st.theta, L.off_table / sizeof(float), 0.0f, c->stream);
    if (e == hipSuccess && n_layers > 0) {
        uint64_t nc = 0;
        build_layer_tables(N, n_layers, cfg->gap_scope == GA_GAP_LAYER ? cfg->host_layer_sizes : nullptr,
                           &c->host_chunks, &c->host_spans, &nc);
        ga::LayerChunk* dchunks = reinterpret_cast<ga::LayerChunk*>(base + L.off_chunks);
        ga::LayerSpan* dspans = reinterpret_cast<ga::LayerSpan*>(base + L.off_spans);
        c->layers.chunks = dchunks;
        c->layers.spans = dspans;
        c->layers.partials = reinterpret_cast<ga::LayerPartial*>(base + L.off_layer_partials);
        c->layers.gaps = reinterpret_cast<float*>(base + L.off_gaps);
        c->layers.n_chunks = (uint32_t)nc;
        c->layers.n_layers = n_layers;
        e = hipMemcpyAsync(dchunks, c->host_chunks.data(), nc * sizeof(ga::LayerChunk), hipMemcpyHostToDevice, c->stream);
        if (e == hipSuccess)
            e = hipMemcpyAsync(dspans, c->host_spans.data(), (size_t)n_layers * sizeof(ga::LayerSpan), hipMemcpyHostToDevice, c->stream);
    }
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&c->rows), ga::kTableCap * sizeof(ga_arrival), hipHostMallocDefault);
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&c->adam_rows), ga::kTableCap * sizeof(ga::AdamRow), hipHostMallocDefault);
    if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&c->grad_rows), ga::kTableCap * sizeof(void*), hipHostMallocDefault);
    if (e == hipSuccess) e = hipEventCreateWithFlags(&c->staged, hipEventDisableTiming);
    if (e != hipSuccess) {
        const int rc = hip_fail(nullptr, e, "create: initial fill or host staging");
        ga_destroy(c);
        return rc;
    }
    *out = c;
    return GA_OK;
}

int ga_create(ga_ctx** out, uint64_t N, uint32_t n_workers, float eta, float gamma, int mode, void* dev_workspace,
              size_t workspace_bytes, void* hip_stream) {
    ga_config cfg;
    ga_config_init(&cfg);
    cfg.N = N;
    cfg.n_workers = n_workers;
    cfg.eta = eta;
    cfg.gamma = gamma;
    cfg.mode = mode;
    return ga_create_ex(out, &cfg, dev_workspace, workspace_bytes, hip_stream);
}

void ga_destroy(ga_ctx* ctx) {
    if (!ctx) return;
    if (ctx->staged_pending) (void)hipEventSynchronize(ctx->staged);
    if (ctx->staged) (void)hipEventDestroy(ctx->staged);
    if (ctx->rows) (void)hipHostFree(ctx->rows);
    if (ctx->adam_rows) (void)hipHostFree(ctx->adam_rows);
    if (ctx->grad_rows) (void)hipHostFree(ctx->grad_rows);
    delete ctx;
}

int ga_set_beta_eps(ga_ctx* ctx, float beta, float eps) {
    if (!ctx) return GA_ERR_ARG;
    if (ctx->k != 0) return fail(ctx, GA_ERR_STATE, "set_beta_eps: only before the first arrival");
    if (!(beta >= 0.f && beta < 1.f)) return fail(ctx, GA_ERR_ARG, "set_beta_eps: beta must be in [0,1)");
    if (!(eps > 0.f) || !std::isfinite(eps)) return fail(ctx, GA_ERR_ARG, "set_beta_eps: eps must be finite and > 0");
    ctx->beta = beta;
    ctx->eps = eps;
    return GA_OK;
}

int ga_set_eta_max(ga_ctx* ctx, float eta_max) {
    if (!ctx) return GA_ERR_ARG;
    if (ctx->k != 0) return fail(ctx, GA_ERR_STATE, "set_eta_max: only before the first arrival");
    if (!(eta_max > 0.f) || !std::isfinite(eta_max)) return fail(ctx, GA_ERR_ARG, "set_eta_max: must be finite and > 0");
    ctx->eta_max = eta_max;
    return GA_OK;
}

int ga_set_lr(ga_ctx* ctx, float eta_k) {
    if (!ctx) return GA_ERR_ARG;
    if (!(eta_k > 0.f) || !std::isfinite(eta_k)) return fail(ctx, GA_ERR_ARG, "set_lr: must be finite and > 0");
    ctx->lr = eta_k;
    return GA_OK;
}

int ga_set_track_gap(ga_ctx* ctx, int on) {
    if (!ctx) return GA_ERR_ARG;
    if (ctx->k != 0) return fail(ctx, GA_ERR_STATE, "set_track_gap: only before the first arrival");
    ctx->track_gap = (on != 0);
    return GA_OK;
}

int ga_set_resident_bytes(ga_ctx* ctx, uint64_t bytes) {
    if (!ctx) return GA_ERR_ARG;
    if (bytes > ((uint64_t)1 << 40)) return fail(ctx, GA_ERR_ARG, "set_resident_bytes: more than 2^40 bytes");
    ctx->st.resident_bytes = bytes;
    return GA_OK;
}

uint64_t ga_get_resident_bytes(const ga_ctx* ctx) { return ctx ? ctx->st.resident_bytes : 0; }

int ga_set_theta(ga_ctx* ctx, const float* dev_theta0) {
    if (!ctx) return GA_ERR_ARG;
    if (!dev_theta0) return fail(ctx, GA_ERR_ARG, "set_theta: source is null");
    if (ctx->k != 0) return fail(ctx, GA_ERR_STATE, "set_theta: only before the first arrival");
    hipError_t e = ga::launch_state_put(ctx->st.theta, ctx->st.rows, dev_theta0, ctx->N, ctx->stream);
    if (e == hipSuccess) e = ga::launch_broadcast_rows(ctx->st.snaps, ctx->st.stride, ctx->W, ctx->st.snap_rows, dev_theta0, ctx->N, ctx->stream);
    return e == hipSuccess ? GA_OK : hip_fail(ctx, e, "set_theta");
}

int ga_apply(ga_ctx* ctx, uint32_t worker_id, const void* dev_grad, int grad_dtype) {
    if (!ctx) return GA_ERR_ARG;
    if (worker_id >= ctx->W) return fail(ctx, GA_ERR_WORKER, "apply: worker %u >= n_workers %u", worker_id, ctx->W);
    if (!dev_grad) return fail(ctx, GA_ERR_ARG, "apply: gradient is null");
    if (grad_dtype != GA_F32 && grad_dtype != GA_BF16) return fail(ctx, GA_ERR_ARG, "apply: unknown gradient dtype %d", grad_dtype);
    if (grad_dtype == GA_F32 && ((uintptr_t)dev_grad & 3u)) return fail(ctx, GA_ERR_ALIGN, "apply: float gradient must be 4-byte aligned");
    if (grad_dtype == GA_BF16 && ((uintptr_t)dev_grad & 1u)) return fail(ctx, GA_ERR_ALIGN, "apply: bfloat16 gradient must be 2-byte aligned");
    return apply_one(ctx, worker_id, dev_grad, grad_dtype, is_gap_mode(ctx->mode) || ctx->track_gap, ctx->lr);
}

int ga_run_schedule(ga_ctx* ctx, const uint32_t* host_schedule, uint64_t T, const ga_grad_source* src) {
    return ga_run_schedule_lr(ctx, host_schedule, T, src, nullptr);
}

static int run_schedule_checked(ga_ctx* ctx, const uint32_t* host_schedule, uint64_t T, const ga_grad_source* src,
                                const float* host_eta);

// Persistent path: the table of a chunk of the schedule is planned on the host, uploaded, and replayed by
// one launch; with gradient buffers the table also names the buffer of every arrival.
// queue_grads != nullptr: one device buffer per arrival, given by the caller (src is then not used).
static int run_persistent(ga_ctx* ctx, const uint32_t* host_schedule, uint64_t T, const ga_grad_source* src,
                          const float* host_eta, const void* const* queue_grads = nullptr, int queue_dtype = GA_F32) {
    const bool buffers = queue_grads || src->kind == GA_SRC_BUFFERS;
    const int grad_dtype = queue_grads ? queue_dtype : src->dtype;
    ga_grad_source none{};
    const ga::RunConst rcst = run_const(ctx, queue_grads ? &none : src);
    for (uint64_t done = 0; done < T;) {
        const uint32_t n = (uint32_t)((T - done < ga::kTableCap) ? (T - done) : ga::kTableCap);
        std::vector<uint64_t> iter_after = ctx->iter;
        std::vector<uint64_t> taus(n);
        hipError_t e = hipSuccess;
        if (ctx->staged_pending) {               // the previous upload from the staging rows must have finished
            e = hipEventSynchronize(ctx->staged);
            if (e != hipSuccess) return hip_fail(ctx, e, "table staging");
            ctx->staged_pending = false;
        }
        plan(n, host_schedule + done, ctx->k, iter_after.data(), ctx->mode, ctx->lr, ctx->beta, ctx->rows, taus.data(),
             host_eta ? host_eta + done : nullptr);
        e = hipMemcpyAsync(ctx->dev_table, ctx->rows, (size_t)n * sizeof(ga_arrival), hipMemcpyHostToDevice, ctx->stream);
        if (e != hipSuccess) return hip_fail(ctx, e, "table upload");
        if (ctx->family == GA_FAMILY_ADAM) {
            for (uint32_t a = 0; a < n; ++a) {
                ctx->adam_rows[a].inv_bc1 = inverse_bias_correction(ctx->beta1, ctx->k + a + 1);
                ctx->adam_rows[a].inv_bc2 = inverse_bias_correction(ctx->beta2, ctx->k + a + 1);
            }
            e = hipMemcpyAsync(ctx->dev_adam_table, ctx->adam_rows, (size_t)n * sizeof(ga::AdamRow), hipMemcpyHostToDevice, ctx->stream);
            if (e != hipSuccess) return hip_fail(ctx, e, "table upload");
        }
        if (buffers) {
            for (uint32_t a = 0; a < n; ++a) {     // the arrival at master step k + a + 1
                if (queue_grads) {
                    ctx->grad_rows[a] = queue_grads[done + a];
                    continue;
                }
                const uint32_t w = host_schedule[done + a];
                const uint64_t b = (src->pick == GA_PICK_BY_WORKER) ? w % src->n_bufs : (ctx->k + a) % src->n_bufs;
                ctx->grad_rows[a] = src->host_dev_bufs[b];
            }
            e = hipMemcpyAsync(ctx->dev_grad_table, ctx->grad_rows, (size_t)n * sizeof(void*), hipMemcpyHostToDevice, ctx->stream);
            if (e != hipSuccess) return hip_fail(ctx, e, "table upload");
        }
        e = hipEventRecord(ctx->staged, ctx->stream);
        if (e != hipSuccess) return hip_fail(ctx, e, "table staging");
        ctx->staged_pending = true;
        if (buffers)
            e = ga::launch_batched(ctx->st, ctx->N, ctx->family, ctx->dev_table, ctx->dev_adam_table, n, ctx->k,
                                   ctx->dev_grad_table, grad_dtype, ctx->mode, ctx->nesterov, keeps_m(ctx), rcst, ctx->stream);
        else
            e = ga::launch_persistent(ctx->st, ctx->N, ctx->family, ctx->dev_table, ctx->dev_adam_table, n, ctx->k, src->dev_a,
                                      src->dev_theta_star, ctx->mode, ctx->nesterov, keeps_m(ctx), rcst, ctx->stream);
        if (e != hipSuccess) return hip_fail(ctx, e, "persistent launch");
        for (const uint64_t tau : taus) record_delay(ctx, tau);
        ctx->iter.swap(iter_after);
        ctx->k += n;
        done += n;
    }
    return GA_OK;
}


int ga_run_schedule_lr(ga_ctx* ctx, const uint32_t* host_schedule, uint64_t T, const ga_grad_source* src,
                       const float* host_eta) {
    if (!ctx) return GA_ERR_ARG;
    const int rc = run_schedule_checked(ctx, host_schedule, T, src, host_eta);
    ctx->layer_sums_ready = false;   // nothing prepared on the device outlives the call
    return rc;
}

static int run_schedule_checked(ga_ctx* ctx, const uint32_t* host_schedule, uint64_t T, const ga_grad_source* src,
                                const float* host_eta) {
    if (!src || (T > 0 && !host_schedule)) return fail(ctx, GA_ERR_ARG, "run_schedule: null argument");
    if (host_eta)
        for (uint64_t a = 0; a < T; ++a)
            if (!(host_eta[a] > 0.f) || !std::isfinite(host_eta[a]))
                return fail(ctx, GA_ERR_ARG, "run_schedule: eta[%llu] must be finite and > 0", (unsigned long long)a);
    for (uint64_t a = 0; a < T; ++a)
        if (host_schedule[a] >= ctx->W)
            return fail(ctx, GA_ERR_WORKER, "run_schedule: schedule[%llu] = %u >= n_workers %u", (unsigned long long)a, host_schedule[a], ctx->W);

    if (src->kind == GA_SRC_BUFFERS) {
        if (!src->host_dev_bufs || src->n_bufs == 0) return fail(ctx, GA_ERR_ARG, "run_schedule: no gradient buffers");
        if (src->dtype != GA_F32 && src->dtype != GA_BF16) return fail(ctx, GA_ERR_ARG, "run_schedule: unknown gradient dtype");
        if (src->pick != GA_PICK_BY_WORKER && src->pick != GA_PICK_BY_ARRIVAL) return fail(ctx, GA_ERR_ARG, "run_schedule: unknown pick rule");
        const uintptr_t need = src->dtype == GA_F32 ? 3u : 1u;
        for (uint32_t b = 0; b < src->n_bufs; ++b)
            if (!src->host_dev_bufs[b] || ((uintptr_t)src->host_dev_bufs[b] & need))
                return fail(ctx, GA_ERR_ARG, "run_schedule: gradient buffer %u is null or misaligned", b);
        if (src->persistent) {
            if (ctx->gap_scope != GA_GAP_PARAMETER)
                return fail(ctx, GA_ERR_ARG, "run_schedule: the persistent kernel exists for the parameter-wise Gap only");
            const uintptr_t vec = src->dtype == GA_F32 ? 15u : 7u;
            for (uint32_t b = 0; b < src->n_bufs; ++b)
                if ((uintptr_t)src->host_dev_bufs[b] & vec)
                    return fail(ctx, GA_ERR_ALIGN, "run_schedule: with persistent set, gradient buffer %u must be aligned to four values", b);
            return run_persistent(ctx, host_schedule, T, src, host_eta);
        }
        const bool write_snap = is_gap_mode(ctx->mode) || ctx->track_gap;
        for (uint64_t a = 0; a < T; ++a) {
            const uint32_t w = host_schedule[a];
            const uint64_t b = (src->pick == GA_PICK_BY_WORKER) ? w % src->n_bufs : ctx->k % src->n_bufs;
            const int64_t next = (a + 1 < T) ? (int64_t)host_schedule[a + 1] : -1;
            const int rc = apply_one(ctx, w, src->host_dev_bufs[b], src->dtype, write_snap, host_eta ? host_eta[a] : ctx->lr, next);
            if (rc != GA_OK) return rc;
        }
        return GA_OK;
    }

    if (src->kind != GA_SRC_QUADRATIC_NOISE) return fail(ctx, GA_ERR_ARG, "run_schedule: unknown source kind %d", src->kind);
    int rc = check_quadratic_source(ctx, src);
    if (rc != GA_OK) return rc;
    const ga::RunConst rcst = run_const(ctx, src);

    if (src->persistent && ctx->gap_scope != GA_GAP_PARAMETER)
        return fail(ctx, GA_ERR_ARG, "run_schedule: the persistent kernel exists for the parameter-wise Gap only");

    if (!src->persistent) {
        // one gradient launch and one update launch per arrival; the worker reads its snapshot,
        // so the snapshot is written in every mode
        if (!src->dev_scratch_g || ((uintptr_t)src->dev_scratch_g & 15u))
            return fail(ctx, GA_ERR_ARG, "run_schedule: dev_scratch_g is null or not 16-byte aligned");
        for (uint64_t a = 0; a < T; ++a) {
            const uint32_t w = host_schedule[a];
            const hipError_t e = ga::launch_quadratic_gradient(ctx->st, ctx->N, w, src->dev_a, src->dev_theta_star,
                                                               ctx->k + 1, rcst, src->dev_scratch_g, ctx->stream);
            if (e != hipSuccess) return hip_fail(ctx, e, "gradient launch");
            const int64_t next = (a + 1 < T) ? (int64_t)host_schedule[a + 1] : -1;
            rc = apply_one(ctx, w, src->dev_scratch_g, GA_F32, true, host_eta ? host_eta[a] : ctx->lr, next);
            if (rc != GA_OK) return rc;
        }
        return GA_OK;
    }

    return run_persistent(ctx, host_schedule, T, src, host_eta);
}

int ga_apply_queue(ga_ctx* ctx, uint64_t n, const uint32_t* host_workers, const void* const* host_dev_grads,
                   int grad_dtype) {
    if (!ctx) return GA_ERR_ARG;
    if (n == 0) return GA_OK;
    if (!host_workers || !host_dev_grads) return fail(ctx, GA_ERR_ARG, "apply_queue: null argument");
    if (grad_dtype != GA_F32 && grad_dtype != GA_BF16) return fail(ctx, GA_ERR_ARG, "apply_queue: unknown gradient dtype");
    if (ctx->gap_scope != GA_GAP_PARAMETER)
        return fail(ctx, GA_ERR_ARG, "apply_queue: the persistent kernel exists for the parameter-wise Gap only");
    const uintptr_t vec = grad_dtype == GA_F32 ? 15u : 7u;
    for (uint64_t a = 0; a < n; ++a) {
        if (host_workers[a] >= ctx->W)
            return fail(ctx, GA_ERR_WORKER, "apply_queue: workers[%llu] = %u >= n_workers %u", (unsigned long long)a, host_workers[a], ctx->W);
        if (!host_dev_grads[a]) return fail(ctx, GA_ERR_ARG, "apply_queue: gradient %llu is null", (unsigned long long)a);
        if ((uintptr_t)host_dev_grads[a] & vec)
            return fail(ctx, GA_ERR_ALIGN, "apply_queue: gradient %llu must be aligned to four values", (unsigned long long)a);
    }
    return run_persistent(ctx, host_workers, n, nullptr, nullptr, host_dev_grads, grad_dtype);
}

int ga_quadratic_gradient(ga_ctx* ctx, uint32_t worker_id, const ga_grad_source* src, float* dev_g_out) {
    if (!ctx) return GA_ERR_ARG;
    if (!src || src->kind != GA_SRC_QUADRATIC_NOISE) return fail(ctx, GA_ERR_ARG, "quadratic_gradient: source must be GA_SRC_QUADRATIC_NOISE");
    if (worker_id >= ctx->W) return fail(ctx, GA_ERR_WORKER, "quadratic_gradient: worker %u >= n_workers %u", worker_id, ctx->W);
    if (!dev_g_out || ((uintptr_t)dev_g_out & 15u)) return fail(ctx, GA_ERR_ALIGN, "quadratic_gradient: output is null or not 16-byte aligned");
    const int rc = check_quadratic_source(ctx, src);
    if (rc != GA_OK) return rc;
    const hipError_t e = ga::launch_quadratic_gradient(ctx->st, ctx->N, worker_id, src->dev_a, src->dev_theta_star,
                                                       ctx->k + 1, run_const(ctx, src), dev_g_out, ctx->stream);
    return e == hipSuccess ? GA_OK : hip_fail(ctx, e, "gradient launch");
}

static int check_diagnostics(ga_ctx* ctx, uint32_t worker_id, const void* out) {
    if (!out) return fail(ctx, GA_ERR_ARG, "diagnostics: output is null");
    if (worker_id >= ctx->W) return fail(ctx, GA_ERR_WORKER, "diagnostics: worker %u >= n_workers %u", worker_id, ctx->W);
    if (!keeps_m(ctx)) return fail(ctx, GA_ERR_STATE, "diagnostics: m is not maintained in this mode (enable gap tracking)");
    return GA_OK;
}

int ga_diagnostics(ga_ctx* ctx, uint32_t worker_id, ga_diag* host_out) {
    if (!ctx) return GA_ERR_ARG;
    const int rc = check_diagnostics(ctx, worker_id, host_out);
    if (rc != GA_OK) return rc;
    hipError_t e = ga::launch_diagnostics(ctx->st, ctx->N, worker_id, inverse_bias_correction(ctx->beta, ctx->k),
                                          ctx->eta_max, ctx->eps, ctx->dev_partials, nullptr, ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "diagnostics launch");
    ga::DiagPartial total;
    e = hipMemcpyAsync(&total, ctx->dev_partials + ga::kDiagMaxBlocks, sizeof total, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "diagnostics readback");
    const double n = (double)ctx->N;
    host_out->mean_graw = total.sum_graw / n;
    host_out->frac_gt1 = (double)total.n_gt1 / n;
    host_out->frac_gt0 = (double)total.n_gt0 / n;
    host_out->n_nonfinite = total.n_bad;
    return GA_OK;
}

int ga_diagnostics_async(ga_ctx* ctx, uint32_t worker_id, ga_diag* dev_out) {
    if (!ctx) return GA_ERR_ARG;
    const int rc = check_diagnostics(ctx, worker_id, dev_out);
    if (rc != GA_OK) return rc;
    if ((uintptr_t)dev_out & 7u) return fail(ctx, GA_ERR_ALIGN, "diagnostics_async: output must be 8-byte aligned");
    const hipError_t e = ga::launch_diagnostics(ctx->st, ctx->N, worker_id, inverse_bias_correction(ctx->beta, ctx->k),
                                                ctx->eta_max, ctx->eps, ctx->dev_partials, dev_out, ctx->stream);
    return e == hipSuccess ? GA_OK : hip_fail(ctx, e, "diagnostics launch");
}

int ga_gap_statistics_static(const float* dev_theta, const float* dev_snapshot, const float* dev_m, uint64_t N,
                             uint64_t k, float beta, float eta_max, float eps, ga_diag* dev_out, void* hip_stream) {
    if (!dev_theta || !dev_snapshot || !dev_m || !dev_out) return fail(nullptr, GA_ERR_ARG, "gap_statistics_static: null argument");
    if (N == 0) return fail(nullptr, GA_ERR_ARG, "gap_statistics_static: N must be positive");
    if (N > GA_STATIC_MAX_N)
        return fail(nullptr, GA_ERR_ARG, "gap_statistics_static: N = %llu is beyond the maximum of %llu parameters",
                    (unsigned long long)N, (unsigned long long)GA_STATIC_MAX_N);
    if (!(beta >= 0.f && beta < 1.f) || !(eps > 0.f) || !std::isfinite(eps) || !(eta_max > 0.f) || !std::isfinite(eta_max))
        return fail(nullptr, GA_ERR_ARG, "gap_statistics_static: beta must be in [0,1), eps and eta_max finite and > 0");
    if (((uintptr_t)dev_theta | (uintptr_t)dev_snapshot | (uintptr_t)dev_m) & 15u)
        return fail(nullptr, GA_ERR_ALIGN, "gap_statistics_static: the arrays must be 16-byte aligned");
    if ((uintptr_t)dev_out & 7u) return fail(nullptr, GA_ERR_ALIGN, "gap_statistics_static: output must be 8-byte aligned");
    const hipError_t e = ga::launch_diagnostics_static(dev_theta, dev_snapshot, dev_m, N, inverse_bias_correction(beta, k),
                                                       eta_max, eps, dev_out, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? GA_OK : hip_fail(nullptr, e, "gap_statistics_static");
}

int ga_get_theta(ga_ctx* ctx, float* dev_dst) { return copy_out(ctx, dev_dst, ctx ? ctx->st.theta : nullptr); }
int ga_get_v(ga_ctx* ctx, float* dev_dst) { return copy_out(ctx, dev_dst, ctx ? ctx->st.v : nullptr); }
int ga_get_m(ga_ctx* ctx, float* dev_dst) { return copy_out(ctx, dev_dst, ctx ? ctx->st.m : nullptr); }
int ga_get_snapshot(ga_ctx* ctx, uint32_t worker_id, float* dev_dst) {
    if (!ctx) return GA_ERR_ARG;
    if (worker_id >= ctx->W) return fail(ctx, GA_ERR_WORKER, "get_snapshot: worker %u >= n_workers %u", worker_id, ctx->W);
    return copy_out(ctx, dev_dst, ctx->st.snaps + (uint64_t)worker_id * ctx->st.stride);
}
int ga_put_theta(ga_ctx* ctx, const float* dev_src) { return copy_in(ctx, ctx ? ctx->st.theta : nullptr, dev_src); }
int ga_put_v(ga_ctx* ctx, const float* dev_src) { return copy_in(ctx, ctx ? ctx->st.v : nullptr, dev_src); }
int ga_put_m(ga_ctx* ctx, const float* dev_src) { return copy_in(ctx, ctx ? ctx->st.m : nullptr, dev_src); }
int ga_put_snapshot(ga_ctx* ctx, uint32_t worker_id, const float* dev_src) {
    if (!ctx) return GA_ERR_ARG;
    if (worker_id >= ctx->W) return fail(ctx, GA_ERR_WORKER, "put_snapshot: worker %u >= n_workers %u", worker_id, ctx->W);
    return copy_in(ctx, ctx->st.snaps + (uint64_t)worker_id * ctx->st.stride, dev_src);
}

static float* array_of(ga_ctx* ctx, int which, uint32_t worker_id, int* status) {
    *status = GA_OK;
    const bool per_worker = (which == GA_ARR_SNAPSHOT || which == GA_ARR_WORKER_V);
    if (per_worker && worker_id >= ctx->W) {
        *status = fail(ctx, GA_ERR_WORKER, "array access: worker %u >= n_workers %u", worker_id, ctx->W);
        return nullptr;
    }
    switch (which) {
        case GA_ARR_THETA: return ctx->st.theta;
        case GA_ARR_V: return ctx->st.v;
        case GA_ARR_M: return ctx->st.m;
        case GA_ARR_SNAPSHOT: return ctx->st.snaps + (uint64_t)worker_id * ctx->st.stride;
        case GA_ARR_WORKER_V:
            if (ctx->st.worker_v) return ctx->st.worker_v + (uint64_t)worker_id * ctx->st.stride;
            break;
        case GA_ARR_ADAM_V2:
            if (ctx->st.v2) return ctx->st.v2;
            break;
        default: break;
    }
    *status = fail(ctx, GA_ERR_ARG, "array access: this context has no array %d", which);
    return nullptr;
}

int ga_get_array(ga_ctx* ctx, int which, uint32_t worker_id, float* dev_dst) {
    if (!ctx) return GA_ERR_ARG;
    int rc;
    float* p = array_of(ctx, which, worker_id, &rc);
    return p ? copy_out(ctx, dev_dst, p) : rc;
}

int ga_put_array(ga_ctx* ctx, int which, uint32_t worker_id, const float* dev_src) {
    if (!ctx) return GA_ERR_ARG;
    int rc;
    float* p = array_of(ctx, which, worker_id, &rc);
    return p ? copy_in(ctx, p, dev_src) : rc;
}

int ga_get_layer_gaps(ga_ctx* ctx, float* host_out, uint32_t max_n) {
    if (!ctx) return GA_ERR_ARG;
    if (!host_out && max_n > 0) return fail(ctx, GA_ERR_ARG, "get_layer_gaps: output is null");
    if (ctx->gap_scope == GA_GAP_PARAMETER) return fail(ctx, GA_ERR_STATE, "get_layer_gaps: the context uses the parameter-wise Gap");
    if (ctx->k == 0) return fail(ctx, GA_ERR_STATE, "get_layer_gaps: no arrival yet");
    const uint32_t n = ctx->layers.n_layers < max_n ? ctx->layers.n_layers : max_n;
    hipError_t e = hipMemcpyAsync(host_out, ctx->layers.gaps, (size_t)n * sizeof(float), hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    return e == hipSuccess ? GA_OK : hip_fail(ctx, e, "get_layer_gaps");
}

uint64_t ga_step(const ga_ctx* ctx) { return ctx ? ctx->k : 0; }

int ga_get_iter(const ga_ctx* ctx, uint64_t* host_iter) {
    if (!ctx || !host_iter) return GA_ERR_ARG;
    std::memcpy(host_iter, ctx->iter.data(), ctx->W * sizeof(uint64_t));
    return GA_OK;
}

int ga_get_delays(const ga_ctx* ctx, uint64_t* host_out, uint64_t max_n, uint64_t* n_out) {
    if (!ctx || (max_n > 0 && !host_out)) return GA_ERR_ARG;
    const uint64_t held = ctx->delays.size();
    const uint64_t n = held < max_n ? held : max_n;            // the n most recent, oldest first
    for (uint64_t i = 0; i < n; ++i) host_out[i] = ctx->delays[(ctx->delay_next + (held - n) + i) % held];
    if (n_out) *n_out = held;
    return GA_OK;
}

int ga_get_config(const ga_ctx* ctx, ga_config* out, float* eta_k) {
    if (!ctx || !out) return GA_ERR_ARG;
    ga_config_init(out);
    out->N = ctx->N;
    out->n_workers = ctx->W;
    out->family = ctx->family;
    out->mode = ctx->mode;
    out->eta = ctx->eta_max;
    out->gamma = ctx->gamma;
    out->beta = ctx->beta;
    out->eps = ctx->eps;
    out->adam_beta1 = ctx->beta1;
    out->adam_beta2 = ctx->beta2;
    out->adam_eps = ctx->adam_eps;
    out->track_gap = ctx->track_gap ? 1 : 0;
    out->gap_scope = ctx->gap_scope;
    out->n_layers = ctx->gap_scope == GA_GAP_LAYER ? ctx->layers.n_layers : 0;
    out->host_layer_sizes = nullptr;
    out->nesterov = ctx->nesterov ? 1 : 0;
    if (eta_k) *eta_k = ctx->lr;
    return GA_OK;
}

int ga_set_bookkeeping(ga_ctx* ctx, uint64_t k, const uint64_t* host_iter) {
    if (!ctx) return GA_ERR_ARG;
    if (!host_iter) return fail(ctx, GA_ERR_ARG, "set_bookkeeping: iter is null");
    for (uint32_t w = 0; w < ctx->W; ++w)
        if (host_iter[w] > k) return fail(ctx, GA_ERR_ARG, "set_bookkeeping: iter[%u] is ahead of k", w);
    ctx->k = k;
    ctx->iter.assign(host_iter, host_iter + ctx->W);
    return GA_OK;
}

int ga_box_muller_raw(const uint32_t* dev_xa, const uint32_t* dev_xb, uint64_t n, float* dev_zc, float* dev_zs,
                      void* hip_stream) {
    if (n > 0 && (!dev_xa || !dev_xb || !dev_zc || !dev_zs)) return fail(nullptr, GA_ERR_ARG, "box_muller_raw: null argument");
    const hipError_t e = ga::launch_box_muller_raw(dev_xa, dev_xb, n, dev_zc, dev_zs, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? GA_OK : hip_fail(nullptr, e, "box_muller_raw launch");
}

size_t ga_state_bytes(const ga_ctx* ctx) { return ctx ? ctx->state_bytes : 0; }

int ga_export_state(ga_ctx* ctx, void* dev_dst, size_t bytes, uint64_t* k, uint64_t* host_iter) {
    if (!ctx) return GA_ERR_ARG;
    if (!dev_dst || !k || !host_iter) return fail(ctx, GA_ERR_ARG, "export_state: null argument");
    if (bytes < ctx->state_bytes) return fail(ctx, GA_ERR_ARG, "export_state: buffer has %zu bytes, %zu needed", bytes, ctx->state_bytes);
    const hipError_t e = hipMemcpyAsync(dev_dst, ctx->st.theta, ctx->state_bytes, hipMemcpyDeviceToDevice, ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "export_state copy");
    *k = ctx->k;
    std::memcpy(host_iter, ctx->iter.data(), ctx->W * sizeof(uint64_t));
    return GA_OK;
}

int ga_import_state(ga_ctx* ctx, const void* dev_src, size_t bytes, uint64_t k, const uint64_t* host_iter) {
    if (!ctx) return GA_ERR_ARG;
    if (!dev_src || !host_iter) return fail(ctx, GA_ERR_ARG, "import_state: null argument");
    if (bytes != ctx->state_bytes) return fail(ctx, GA_ERR_ARG, "import_state: checkpoint has %zu bytes, this context %zu", bytes, ctx->state_bytes);
    for (uint32_t w = 0; w < ctx->W; ++w)
        if (host_iter[w] > k) return fail(ctx, GA_ERR_ARG, "import_state: iter[%u] is ahead of k", w);
    const hipError_t e = hipMemcpyAsync(ctx->st.theta, dev_src, ctx->state_bytes, hipMemcpyDeviceToDevice, ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, e, "import_state copy");
    ctx->k = k;
    ctx->iter.assign(host_iter, host_iter + ctx->W);
    return GA_OK;
}

int ga_probe_streams_ex(uint32_t n_read, uint32_t n_write, uint32_t n_resident, int tiled, uint64_t n,
                        const float* const* host_dev_read, float* const* host_dev_write, void* hip_stream) {
    const bool r_ok = n_read == 0 || n_read == 1 || n_read == 2 || n_read == 4 || n_read == 5;
    const bool w_ok = n_write == 0 || n_write == 1 || n_write == 2 || n_write == 4;
    if (!r_ok || !w_ok || n_read + n_write == 0) return fail(nullptr, GA_ERR_ARG, "probe_streams: n_read must be 0, 1, 2, 4 or 5 and n_write 0, 1, 2 or 4, not both 0");
    if (n_resident > 2) return fail(nullptr, GA_ERR_ARG, "probe_streams: n_resident must be 0, 1 or 2");
    if (tiled != 0 && tiled != 1) return fail(nullptr, GA_ERR_ARG, "probe_streams: tiled must be 0 or 1");
    if (n == 0 || (n & 3u)) return fail(nullptr, GA_ERR_ARG, "probe_streams: n must be a positive multiple of 4");
    if ((n_read && !host_dev_read) || (n_write && !host_dev_write)) return fail(nullptr, GA_ERR_ARG, "probe_streams: null pointer table");
    for (uint32_t i = 0; i < n_read; ++i)
        if (!host_dev_read[i] || ((uintptr_t)host_dev_read[i] & 15u)) return fail(nullptr, GA_ERR_ARG, "probe_streams: input %u is null or not 16-byte aligned", i);
    for (uint32_t i = 0; i < n_write; ++i)
        if (!host_dev_write[i] || ((uintptr_t)host_dev_write[i] & 15u)) return fail(nullptr, GA_ERR_ARG, "probe_streams: output %u is null or not 16-byte aligned", i);
    const hipError_t e = ga::launch_probe_streams(n_read, n_write, n_resident, tiled != 0, n, host_dev_read, host_dev_write, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? GA_OK : hip_fail(nullptr, e, "probe_streams launch");
}

int ga_probe_streams(uint32_t n_read, uint32_t n_write, uint64_t n, const float* const* host_dev_read,
                     float* const* host_dev_write, void* hip_stream) {
    return ga_probe_streams_ex(n_read, n_write, 0, 0, n, host_dev_read, host_dev_write, hip_stream);
}

int ga_probe_valu(int op, uint32_t blocks, uint32_t iterations, uint32_t* dev_out, void* hip_stream) {
    if (op < GA_PROBE_FMA || op > GA_PROBE_DIV_FIXUP) return fail(nullptr, GA_ERR_ARG, "probe_valu: unknown op %d", op);
    if (blocks == 0 || blocks > (1u << 20) || !dev_out) return fail(nullptr, GA_ERR_ARG, "probe_valu: blocks must be 1 .. 2^20 and dev_out not null");
    const hipError_t e = ga::launch_probe_valu(op, blocks, iterations, dev_out, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? GA_OK : hip_fail(nullptr, e, "probe_valu launch");
}

int ga_noise_fill(uint64_t seed, uint64_t k, uint64_t j0, uint64_t n, float* dev_out, void* hip_stream) {
    if (n > 0 && !dev_out) return fail(nullptr, GA_ERR_ARG, "noise_fill: output is null");
    const hipError_t e = ga::launch_noise_fill(seed, k, j0, n, dev_out, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? GA_OK : hip_fail(nullptr, e, "noise_fill launch");
}

}  // extern "C"
