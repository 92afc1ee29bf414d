// Test scaffolding (CPU only): the whole library -- host code and kernel sources, the latter compiled for the CPU
// through shim/hip/hip_runtime.h and run by cpu_device.cpp -- driven through one scenario that a test describes in a
// directory of small files; the resulting state is written back for comparison with the oracle.
//
//   driver <directory>
//
// <directory>/scenario.txt: "name value" lines (integers; eta as a decimal).  Binary inputs beside it: sched.bin
// (uint32 worker ids), a.bin / ts.bin (float, quadratic source), bufs.bin (n_bufs x N float or bfloat16 bits),
// layers.bin (uint64 layer sizes), theta0.bin (float, optional start).  Output: state.bin.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <string>
#include <vector>

#include "ga.h"

#define REQUIRE(cond)                                                                              \
    do {                                                                                           \
        if (!(cond)) {                                                                             \
            std::fprintf(stderr, "driver: line %d: %s is false (%s)\n", __LINE__, #cond,           \
                         ga_last_error(ctx));                                                      \
            return 1;                                                                              \
        }                                                                                          \
    } while (0)

static void* device_alloc(size_t bytes) {
    void* p = std::aligned_alloc(256, (bytes + 255) / 256 * 256);
    std::memset(p, 0xA5, (bytes + 255) / 256 * 256);   // nothing may rely on fresh memory being zero
    return p;
}

template <typename T>
static std::vector<T> read_file(const std::string& path, size_t count) {
    std::vector<T> v(count);
    FILE* f = std::fopen(path.c_str(), "rb");
    if (!f || std::fread(v.data(), sizeof(T), count, f) != count) {
        std::fprintf(stderr, "driver: cannot read %zu items from %s\n", count, path.c_str());
        std::exit(3);
    }
    std::fclose(f);
    return v;
}

int main(int argc, char** argv) {
    if (argc != 2) return 2;
    const std::string dir = argv[1];
    std::map<std::string, double> s;
    {
        FILE* f = std::fopen((dir + "/scenario.txt").c_str(), "r");
        if (!f) return 3;
        char name[64];
        double value;
        while (std::fscanf(f, "%63s %lf", name, &value) == 2) s[name] = value;
        std::fclose(f);
    }
    const uint64_t N = (uint64_t)s["N"], T = (uint64_t)s["T"], seed = (uint64_t)s["seed"];
    const uint32_t W = (uint32_t)s["W"], n_bufs = (uint32_t)s["n_bufs"], n_layers = (uint32_t)s["n_layers"];
    // source: 0 quadratic in the persistent kernel, 1 quadratic one arrival per launch, 2 gradient buffers one arrival
    // per launch, 3 gradient buffers in the persistent kernel; the second half of the arrivals of source 2 goes
    // through ga_apply_queue when "queue" is set
    const int source = (int)s["source"], bf16 = (int)s["bf16"];
    ga_ctx* ctx = nullptr;

    ga_config cfg;
    ga_config_init(&cfg);
    cfg.N = N; cfg.n_workers = W; cfg.family = (int)s["family"]; cfg.mode = (int)s["mode"]; cfg.eta = (float)s["eta"];
    cfg.gamma = (float)s["gamma"]; cfg.track_gap = (int)s["track_gap"]; cfg.gap_scope = (int)s["gap_scope"];
    cfg.nesterov = (int)s["nesterov"];
    std::vector<uint64_t> layers;
    if (cfg.gap_scope == GA_GAP_LAYER) {
        layers = read_file<uint64_t>(dir + "/layers.bin", n_layers);
        cfg.n_layers = n_layers;
        cfg.host_layer_sizes = layers.data();
    }
    const size_t ws_bytes = ga_workspace_bytes_ex(&cfg);
    REQUIRE(ws_bytes > 0);
    void* ws = device_alloc(ws_bytes);
    REQUIRE(ga_create_ex(&ctx, &cfg, ws, ws_bytes, nullptr) == GA_OK);
    REQUIRE(ga_set_resident_bytes(ctx, (uint64_t)s["resident_bytes"]) == GA_OK);
    if ((int)s["theta0"]) {   // a start other than zero: theta and every snapshot (Alg. 2: theta^i = theta_0)
        const std::vector<float> theta0 = read_file<float>(dir + "/theta0.bin", N);
        REQUIRE(ga_set_theta(ctx, theta0.data()) == GA_OK);
    }

    const std::vector<uint32_t> sched = read_file<uint32_t>(dir + "/sched.bin", T);
    std::vector<float> a, ts;
    float* scratch_g = nullptr;
    std::vector<void*> bufs;
    std::vector<const void*> buf_table;
    ga_grad_source src{};
    if (source <= 1) {
        a = read_file<float>(dir + "/a.bin", N);
        ts = read_file<float>(dir + "/ts.bin", N);
        scratch_g = (float*)device_alloc(N * sizeof(float));
        src.kind = GA_SRC_QUADRATIC_NOISE; src.dev_a = a.data(); src.dev_theta_star = ts.data(); src.seed = seed;
        src.sigma = (float)s["sigma"]; src.persistent = source == 0; src.dev_scratch_g = scratch_g;
    } else {
        const size_t elt = bf16 ? 2 : 4;
        const std::vector<char> raw = read_file<char>(dir + "/bufs.bin", (size_t)n_bufs * N * elt);
        for (uint32_t b = 0; b < n_bufs; ++b) {
            // exactly N values and no more, so that a read past the end of a buffer is seen
            void* p = std::malloc(N * elt);
            std::memcpy(p, raw.data() + (size_t)b * N * elt, N * elt);
            bufs.push_back(p);
            buf_table.push_back(p);
        }
        src.kind = GA_SRC_BUFFERS; src.host_dev_bufs = buf_table.data(); src.n_bufs = n_bufs;
        src.dtype = bf16 ? GA_BF16 : GA_F32; src.pick = (int)s["pick"]; src.persistent = source == 3;
    }

    const uint64_t cut = T / 3;
    REQUIRE(ga_run_schedule(ctx, sched.data(), cut, &src) == GA_OK);
    if (source == 2 && (int)s["queue"]) {
        std::vector<const void*> grads(T - cut);
        for (uint64_t i = cut; i < T; ++i)
            grads[i - cut] = buf_table[src.pick == GA_PICK_BY_WORKER ? sched[i] % n_bufs : i % n_bufs];
        REQUIRE(ga_apply_queue(ctx, T - cut, sched.data() + cut, grads.data(), src.dtype) == GA_OK);
    } else {
        REQUIRE(ga_run_schedule(ctx, sched.data() + cut, T - cut, &src) == GA_OK);
    }
    REQUIRE(ga_step(ctx) == T);

    FILE* out = std::fopen((dir + "/state.bin").c_str(), "wb");
    REQUIRE(out);
    std::vector<float> row(N);
    auto dump = [&](int which, uint32_t worker) {
        if (ga_get_array(ctx, which, worker, row.data()) != GA_OK) return false;
        std::fwrite(row.data(), sizeof(float), N, out);
        return true;
    };
    const bool keeps_m = cfg.mode == GA_MODE_GA || cfg.mode == GA_MODE_GA_HINGE || cfg.track_gap;
    REQUIRE(dump(GA_ARR_THETA, 0));
    REQUIRE(dump(GA_ARR_V, 0));
    if (keeps_m) {
        REQUIRE(dump(GA_ARR_M, 0));
        for (uint32_t w = 0; w < W; ++w) REQUIRE(dump(GA_ARR_SNAPSHOT, w));
    }
    if (cfg.family == GA_FAMILY_DANA)
        for (uint32_t w = 0; w < W; ++w) REQUIRE(dump(GA_ARR_WORKER_V, w));
    if (cfg.family == GA_FAMILY_ADAM) REQUIRE(dump(GA_ARR_ADAM_V2, 0));
    std::vector<uint64_t> iter(W);
    REQUIRE(ga_get_iter(ctx, iter.data()) == GA_OK);
    std::fwrite(iter.data(), sizeof(uint64_t), W, out);
    if (keeps_m) {
        ga_diag d;
        REQUIRE(ga_diagnostics(ctx, (uint32_t)s["diag_worker"], &d) == GA_OK);
        std::fwrite(&d, sizeof d, 1, out);
        if ((int)s["static_diag"]) {   // the same statistics through the entry point with the static partials
            std::vector<float> theta(N), m(N), snap(N);
            ga_diag d2;
            REQUIRE(ga_get_array(ctx, GA_ARR_THETA, 0, theta.data()) == GA_OK);
            REQUIRE(ga_get_array(ctx, GA_ARR_M, 0, m.data()) == GA_OK);
            REQUIRE(ga_get_array(ctx, GA_ARR_SNAPSHOT, (uint32_t)s["diag_worker"], snap.data()) == GA_OK);
            float* al[3];
            for (int i = 0; i < 3; ++i) al[i] = (float*)device_alloc(N * sizeof(float));
            std::memcpy(al[0], theta.data(), N * 4); std::memcpy(al[1], snap.data(), N * 4); std::memcpy(al[2], m.data(), N * 4);
            REQUIRE(ga_gap_statistics_static(al[0], al[1], al[2], N, T, cfg.beta, cfg.eta, cfg.eps, &d2, nullptr) == GA_OK);
            REQUIRE(std::memcmp(&d, &d2, sizeof d) == 0);
            for (auto p : al) std::free(p);
        }
    }
    if (cfg.gap_scope != GA_GAP_PARAMETER) {
        const uint32_t nl = cfg.gap_scope == GA_GAP_GLOBAL ? 1 : n_layers;
        std::vector<float> gaps(nl);
        REQUIRE(ga_get_layer_gaps(ctx, gaps.data(), nl) == GA_OK);
        std::fwrite(gaps.data(), sizeof(float), nl, out);
    }
    std::fclose(out);
    ga_destroy(ctx);
    ctx = nullptr;
    for (void* p : bufs) std::free(p);
    std::free(scratch_g);
    std::free(ws);
    std::puts("cpu device driver ok");
    return 0;
}
