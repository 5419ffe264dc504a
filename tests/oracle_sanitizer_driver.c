/* Drives the CPU oracle through all of its modes on small ragged sizes; built with
 * -fsanitize=address,undefined by test_oracle_pins.py (host code only, no GPU involved). */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "asyncmesh_oracle.c"
int main(void) {
    const uint64_t ns[] = {1, 3, 255, 257, 5003};
    for (int c = 0; c < 5; ++c) for (uint32_t opt = 0; opt < 3; ++opt) for (uint32_t strat = 0; strat < 2; ++strat) {
        amo_config cfg; memset(&cfg, 0, sizeof cfg);
        cfg.n = ns[c]; cfg.mu0 = 7; cfg.replicas = 3; cfg.delay = 2; cfg.avg_interval = 2; cfg.optimizer = opt;
        cfg.fraction = 0.3; cfg.seed = 5; cfg.beta1 = 0.9; cfg.beta2 = 0.999; cfg.eps = 1e-8; cfg.weight_decay = 0.01;
        cfg.gamma = 0.9; cfg.lookahead = 1; cfg.correction = 1 + (c & 1); cfg.fwd_bf16 = c & 1; cfg.grad_bf16 = 0;
        cfg.momentum_decay = 0.004; cfg.granule = strat ? 1 : (c == 2 ? 32 : 1); cfg.msg_dtype = c % 3; cfg.stratified = strat;
        amo_state *s = amo_create(&cfg);
        float *g[3]; const void *gp[3];
        for (int i = 0; i < 3; ++i) { g[i] = malloc(sizeof(float) * cfg.n); for (uint64_t k = 0; k < cfg.n; ++k) g[i][k] = 1e-3f * (float)((k * 7 + i) % 11) - 5e-3f; gp[i] = g[i]; }
        for (uint64_t k = 0; k < cfg.n; ++k) for (int i = 0; i < 3; ++i) amo_w(s, i)[k] = 0.02f * (float)(k % 5);
        float rs[3] = {1.f, 0.5f, 2.f};
        for (uint64_t t = 1; t <= 9; ++t) {
            int rc;
            if (t % 3 == 0) rc = amo_step_masked(s, t, gp, 1e-3, 0.5, 1.0, rs, 0x5);
            else if (t % 3 == 1) rc = amo_step(s, t, gp, 1e-3, 0.5, 1.0);
            else rc = amo_sparse_average(s, t, 0.5);
            if (rc) { printf("rc %d\n", rc); return 1; }
            if (t == 4) amo_set_delay(s, 1);
        }
        double a, b; amo_ema_variance(s, &a, &b);
        printf("n=%llu opt=%u strat=%u cons=%g var=%g\n", (unsigned long long)cfg.n, opt, strat, amo_consensus_error(s), a);
        uint64_t out[64]; amo_subset(5, 3, 0, 200, 0.3, 1, strat, out, 64);
        for (int i = 0; i < 3; ++i) free(g[i]);
        amo_destroy(s);
    }
    return 0;
}
