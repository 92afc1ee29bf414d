// Test scaffolding (CPU only): drives the host side of libga (ga_host.cpp linked against fake_runtime.cpp and fake_launchers.cpp) through
// one scenario and writes what the host decided -- the schedule, k, iter[], the delay log and one record per
// arrival as handed to the launchers -- to a binary file that tests/test_host_sim.py compares with the oracle.
//
//   driver <out file> <family> <mode> <gap scope> <W> <T> <seed>
//
// The T arrivals are split over the entry points: ga_run_schedule with the in-kernel quadratic source (parameter-wise
// Gap only), ga_apply one arrival at a time, ga_run_schedule_lr with gradient buffers and a step size per arrival,
// ga_apply_queue (parameter-wise Gap only); a checkpoint is exported and imported on the way, and calls with wrong
// arguments in between must fail and change nothing.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "ga.h"

struct LoggedArrival {
    uint32_t worker;
    float tau, lr, inv_bc_prev;
    int path;
};
extern std::vector<LoggedArrival> g_rows;

#define REQUIRE(cond)                                                                  \
    do {                                                                               \
        if (!(cond)) {                                                                 \
            std::fprintf(stderr, "driver: line %d: %s is false\n", __LINE__, #cond);   \
            return 1;                                                                  \
        }                                                                              \
    } while (0)

static void* device_alloc(size_t bytes) { return std::aligned_alloc(256, (bytes + 255) / 256 * 256); }

int main(int argc, char** argv) {
    if (argc != 8) return 2;
    const char* out_path = argv[1];
    const int family = std::atoi(argv[2]), mode = std::atoi(argv[3]), scope = std::atoi(argv[4]);
    const uint32_t W = (uint32_t)std::atoi(argv[5]);
    const uint64_t T = std::strtoull(argv[6], nullptr, 10), seed = std::strtoull(argv[7], nullptr, 10);
    const uint64_t N = 1000;
    const float eta = 0.05f;

    std::vector<uint32_t> sched(T);
    REQUIRE(ga_simulate_schedule(W, T, GA_DIST_EXP, 1.0, seed, sched.data()) == GA_OK);

    ga_config cfg;
    ga_config_init(&cfg);
    cfg.N = N; cfg.n_workers = W; cfg.family = family; cfg.mode = mode; cfg.eta = eta; cfg.gap_scope = scope;
    const uint64_t layer_sizes[2] = {300, 700};
    if (scope == GA_GAP_LAYER) { cfg.n_layers = 2; cfg.host_layer_sizes = layer_sizes; }
    const size_t ws_bytes = ga_workspace_bytes_ex(&cfg);
    REQUIRE(ws_bytes > 0);
    void* ws = device_alloc(ws_bytes);
    std::memset(ws, 0, ws_bytes);
    ga_ctx* ctx = nullptr;
    REQUIRE(ga_create_ex(&ctx, &cfg, (char*)ws + 4, ws_bytes, nullptr) == GA_ERR_ALIGN);
    REQUIRE(ga_create_ex(&ctx, &cfg, ws, ws_bytes - 1, nullptr) == GA_ERR_ALIGN);   // short workspace
    REQUIRE(ga_create_ex(&ctx, &cfg, ws, ws_bytes, nullptr) == GA_OK && ctx);

    std::vector<float> a(N, 0.5f), ts(N, 1.0f);
    float* bufs[3];
    for (auto& b : bufs) b = (float*)device_alloc(N * sizeof(float));
    const void* buf_table[3] = {bufs[0], bufs[1], bufs[2]};
    ga_grad_source quad{};
    quad.kind = GA_SRC_QUADRATIC_NOISE; quad.dev_a = a.data(); quad.dev_theta_star = ts.data(); quad.seed = seed;
    quad.sigma = 0.01f; quad.persistent = 1;
    ga_grad_source from_bufs{};
    from_bufs.kind = GA_SRC_BUFFERS; from_bufs.host_dev_bufs = buf_table; from_bufs.n_bufs = 3; from_bufs.dtype = GA_F32;
    from_bufs.pick = GA_PICK_BY_ARRIVAL;

    const bool per_parameter = scope == GA_GAP_PARAMETER;
    uint64_t done = 0;
    const uint64_t part = T / 4;
    // 1: persistent quadratic source
    if (per_parameter) {
        REQUIRE(ga_run_schedule(ctx, sched.data(), part, &quad) == GA_OK);
        done = part;
    }
    REQUIRE(ga_step(ctx) == done);
    // wrong arguments change nothing
    REQUIRE(ga_apply(ctx, W, bufs[0], GA_F32) == GA_ERR_WORKER);
    REQUIRE(ga_apply(ctx, 0, nullptr, GA_F32) == GA_ERR_ARG);
    REQUIRE(ga_apply(ctx, 0, bufs[0], 7) == GA_ERR_ARG);
    if (done > 0) REQUIRE(ga_set_beta_eps(ctx, 0.99f, 1e-6f) == GA_ERR_STATE);
    REQUIRE(ga_step(ctx) == done);
    // 2: one arrival per call
    for (; done < 2 * part; ++done) REQUIRE(ga_apply(ctx, sched[done], bufs[done % 3], GA_F32) == GA_OK);
    // checkpoint out and in again
    {
        const size_t sb = ga_state_bytes(ctx);
        void* ck = device_alloc(sb);
        uint64_t k = 0;
        std::vector<uint64_t> it(W);
        REQUIRE(ga_export_state(ctx, ck, sb - 1, &k, it.data()) == GA_ERR_ARG);
        REQUIRE(ga_export_state(ctx, ck, sb, &k, it.data()) == GA_OK && k == done);
        std::vector<uint64_t> bad = it;
        bad[0] = k + 1;
        REQUIRE(ga_import_state(ctx, ck, sb, k, bad.data()) == GA_ERR_ARG);
        REQUIRE(ga_import_state(ctx, ck, sb, k, it.data()) == GA_OK);
        std::free(ck);
    }
    // 3: gradient buffers with a step size per arrival (one launch per arrival)
    {
        const uint64_t n = part;
        std::vector<float> etas(n);
        for (uint64_t i = 0; i < n; ++i) etas[i] = eta * (1.0f + (float)(i % 7) / 8.0f);
        REQUIRE(ga_run_schedule_lr(ctx, sched.data() + done, n, &from_bufs, etas.data()) == GA_OK);
        etas[n / 2] = -1.0f;
        REQUIRE(ga_run_schedule_lr(ctx, sched.data() + done, n, &from_bufs, etas.data()) == GA_ERR_ARG);
        done += n;
        REQUIRE(ga_step(ctx) == done);
    }
    // 4: a queue of arrivals with their own gradients
    if (per_parameter) {
        const uint64_t n = T - done;
        std::vector<const void*> grads(n);
        for (uint64_t i = 0; i < n; ++i) grads[i] = bufs[i % 3];
        REQUIRE(ga_apply_queue(ctx, n, sched.data() + done, grads.data(), GA_F32) == GA_OK);
        done += n;
    } else {
        for (; done < T; ++done) REQUIRE(ga_apply(ctx, sched[done], bufs[done % 3], GA_F32) == GA_OK);
    }
    REQUIRE(ga_step(ctx) == T && g_rows.size() == T);

    std::vector<uint64_t> iter(W);
    REQUIRE(ga_get_iter(ctx, iter.data()) == GA_OK);
    uint64_t kept = 0;
    REQUIRE(ga_get_delays(ctx, nullptr, 0, &kept) == GA_OK);
    std::vector<uint64_t> delays(kept);
    REQUIRE(ga_get_delays(ctx, delays.data(), kept, nullptr) == GA_OK);
    ga_diag d;
    const bool gap_mode = mode == GA_MODE_GA || mode == GA_MODE_GA_HINGE;   // Alg. 14's m exists without tracking
    REQUIRE(ga_diagnostics(ctx, 0, &d) == (gap_mode ? GA_OK : GA_ERR_STATE));
    REQUIRE(ga_diagnostics(ctx, W, &d) == GA_ERR_WORKER);

    FILE* f = std::fopen(out_path, "wb");
    REQUIRE(f);
    const uint64_t head[3] = {T, kept, (uint64_t)W};
    std::fwrite(head, sizeof head, 1, f);
    std::fwrite(sched.data(), sizeof(uint32_t), T, f);
    std::fwrite(iter.data(), sizeof(uint64_t), W, f);
    std::fwrite(delays.data(), sizeof(uint64_t), kept, f);
    std::fwrite(g_rows.data(), sizeof(LoggedArrival), g_rows.size(), f);
    std::fclose(f);

    ga_destroy(ctx);
    for (auto& b : bufs) std::free(b);
    std::free(ws);
    std::puts("host driver ok");
    return 0;
}
