/* The C ABI used from plain C99 (no Python, no C++): a host-only context builds and exports a plan,
 * resolves slots, fits the latency predictor and runs one planner invocation.  Prints "ok" and
 * returns 0 when every check holds.  Built and run by tests/test_c_abi.py. */
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "taper_admission.h"
#include "taper_attn.h"

#define CHECK(cond)                                                                  \
    do {                                                                             \
        if (!(cond)) {                                                               \
            fprintf(stderr, "%s:%d: %s failed (%s)\n", __FILE__, __LINE__, #cond, taper_last_error()); \
            return 1;                                                                \
        }                                                                            \
    } while (0)

int main(void)
{
    taper_attn_config cfg;
    memset(&cfg, 0, sizeof cfg);
    cfg.n_q_heads = 64;
    cfg.n_kv_heads = 8;
    cfg.head_dim = 128;
    cfg.page_size = 16;
    cfg.scale = 0.088388347f;
    cfg.device = -1; /* host only */
    taper_ctx *ctx = NULL;
    CHECK(taper_create(&cfg, &ctx) == TAPER_OK);

    /* one serial request (40 tokens) and one request with two branches sharing a 20-token prefix */
    enum { S = 3, STRIDE = 4 };
    const int32_t bt[S * STRIDE] = {5, 6, 7, -1, /**/ 1, 2, 3, -1, /**/ 1, 2, 4, 9};
    const int32_t group[S] = {0, 1, 1};
    const int32_t prefix[S] = {40, 20, 20};
    const int32_t suffix[S] = {0, 5, 17};
    taper_plan *plan = NULL;
    CHECK(taper_plan_build(ctx, S, bt, STRIDE, group, prefix, suffix, 16, NULL, NULL, &plan) == TAPER_OK);
    taper_plan_view v;
    CHECK(taper_plan_export(plan, &v) == TAPER_OK);
    CHECK(v.n_seqs == 3 && v.n_groups == 2);
    CHECK(v.ctx_len[0] == 40 && v.ctx_len[1] == 25 && v.ctx_len[2] == 37);
    CHECK(v.n_prefix_pages[1] == 2 && v.n_suffix_pages[1] == 1 && v.n_suffix_pages[2] == 2);
    CHECK(v.tokens_unique == 40 + 20 + 5 + 17 && v.tokens_logical == 40 + 25 + 37);
    int64_t slots[S * 40];
    CHECK(taper_plan_resolve_slots_host(plan, slots, 40) == TAPER_OK);
    CHECK(slots[0] == 5 * 16 && slots[39] == 7 * 16 + 7);
    CHECK(slots[40 + 19] == 2 * 16 + 3 && slots[40 + 20] == 3 * 16 && slots[40 + 25] == -1);
    CHECK(slots[80 + 20] == 4 * 16 && slots[80 + 36] == 9 * 16);
    /* a malformed batch is refused with a status, not a crash */
    const int32_t bad_group[S] = {0, 2, 2};
    taper_plan *none = NULL;
    CHECK(taper_plan_build(ctx, S, bt, STRIDE, bad_group, prefix, suffix, 16, NULL, NULL, &none) == TAPER_EGROUP);
    CHECK(strlen(taper_last_error()) > 0);
    /* device work on a host-only context is refused */
    CHECK(taper_decode_step_attention(ctx, plan, bt, bt, (void *)slots, NULL, NULL) == TAPER_EHIP);
    taper_plan_free(plan);
    taper_destroy(ctx);
    CHECK(taper_branch_blocks(17, 16) == 2 && taper_branch_blocks(0, 16) == 0);

    /* predictor: four observations with an orthogonal design -> a = -4, b = 3, c = 2, MAPE 25 % */
    const double n[4] = {1, 1, 3, 3}, L[4] = {1, 3, 1, 3}, t[4] = {2, 4, 6, 12};
    taper_predictor p;
    double mape = 0;
    CHECK(taper_predictor_fit(4, n, L, t, &p, &mape) == TAPER_OK);
    CHECK(fabs(p.a + 4) < 1e-12 && fabs(p.b - 3) < 1e-12 && fabs(p.c - 2) < 1e-12 && fabs(mape - 25) < 1e-9);

    /* planner: the three-request example (budget 12.4 ms -> grants 0, 2, 2 with 7 evaluations of T) */
    const taper_predictor T = {1.0, 0.1, 0.001};
    const int64_t base[3] = {1000, 2000, 500};
    const double slack[3] = {50, 20, 100};
    const int32_t start[4] = {0, 0, 3, 5};
    const int64_t branch[5] = {2000, 2100, 2200, 500, 600};
    taper_admission_options o;
    memset(&o, 0, sizeof o);
    o.rho = 0.5;
    o.utility_kind = TAPER_UTILITY_LINEAR;
    int32_t granted[3];
    taper_admission_result r;
    CHECK(taper_admit_step(&T, 3, base, slack, start, branch, NULL, NULL, &o, granted, &r) == TAPER_OK);
    CHECK(granted[0] == 0 && granted[1] == 2 && granted[2] == 2 && r.evaluations == 7 && r.admitted == 4);
    CHECK(fabs(r.budget_ms - 12.4) < 1e-12 && fabs(r.t_pred_ms - 10.4) < 1e-9);
    o.rho = 0.0;
    CHECK(taper_admit_step(&T, 3, base, slack, start, branch, NULL, NULL, &o, granted, &r) == TAPER_EINVAL);
    printf("ok\n");
    return 0;
}
