/* A plain C99 client of include/ga.h: host-only entry points and the argument checks of ga_create.
 * Built and run by tests/test_abi_host.py (no GPU needed). */
#include <stdio.h>
#include <string.h>

#include "ga.h"

#define CHECK(cond)                                                  \
    do {                                                             \
        if (!(cond)) {                                               \
            printf("FAILED line %d: %s\n", __LINE__, #cond);         \
            return 1;                                                \
        }                                                            \
    } while (0)

int main(void) {
    uint32_t schedule[64];
    uint64_t iter[4] = {0, 0, 0, 0}, tau[64];
    ga_arrival rows[64];
    ga_config cfg;
    ga_ctx* ctx = (ga_ctx*)0;
    uint64_t sizes[2] = {60, 40};
    int i;

    CHECK(strcmp(ga_version(), "0.1") == 0);
    CHECK(ga_simulate_schedule(4, 64, GA_DIST_EXP, 1.0, 7, schedule) == GA_OK);
    for (i = 0; i < 64; ++i) CHECK(schedule[i] < 4);
    CHECK(ga_delays_from_schedule(4, 64, schedule, 0, iter, tau) == GA_OK);
    CHECK(tau[0] == 1);
    memset(iter, 0, sizeof iter);
    CHECK(ga_plan_arrivals(4, 64, schedule, 0, iter, GA_MODE_SA_STEP, 0.1f, 0.999f, rows) == GA_OK);
    CHECK(rows[0].worker == schedule[0] && rows[0].tau == 1.0f && rows[0].inv_bc_prev == 0.0f);
    CHECK(rows[5].lr == 0.1f / rows[5].tau);

    CHECK(ga_workspace_bytes(0, 4) == 0);
    CHECK(ga_workspace_bytes(100, 4) % 256 == 0);
    ga_config_init(&cfg);
    cfg.N = 100;
    cfg.n_workers = 4;
    cfg.gap_scope = GA_GAP_LAYER;
    cfg.n_layers = 2;
    cfg.host_layer_sizes = sizes;
    CHECK(ga_workspace_bytes_ex(&cfg) > ga_workspace_bytes(100, 4));
    sizes[1] = 41;                                  /* does not sum to N */
    CHECK(ga_workspace_bytes_ex(&cfg) == 0);
    CHECK(ga_create_ex(&ctx, &cfg, (void*)0x7f0000000000, (size_t)1 << 30, (void*)0) == GA_ERR_ARG);
    CHECK(ctx == (ga_ctx*)0);
    CHECK(strstr(ga_last_error((ga_ctx*)0), "layer") != (char*)0);
    CHECK(ga_create(&ctx, 100, 4, 0.1f, 0.9f, GA_MODE_GA, (void*)0, 0, (void*)0) == GA_ERR_ARG);
    CHECK(ga_apply((ga_ctx*)0, 0, (void*)0, GA_F32) == GA_ERR_ARG);
    ga_destroy((ga_ctx*)0);
    printf("c client ok\n");
    return 0;
}
