/* Host-side fuzz of the planning, layout, cost-model and error paths of the C ABI: thousands of
 * random nets through the calls that need no GPU.  Built with AddressSanitizer and
 * UndefinedBehaviorSanitizer by tests/test_host_sanitizers.py; every return code is checked and
 * the sanitizers watch the library's host code. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "mgwfbp.h"
static unsigned long long s = 88172645463325252ULL;
static unsigned long long rnd(void) { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return s; }
static double urand(void) { return (rnd() >> 11) * (1.0 / 9007199254740992.0); }
int main(void)
{
    int it, bad = 0;
    for (it = 0; it < 3000; ++it) {
        int L = 1 + (int)(rnd() % 60), N = 1 + (int)(rnd() % 20), l;
        uint64_t *p = malloc(sizeof(uint64_t) * L);
        double *tb = malloc(sizeof(double) * L);
        uint8_t *merged = malloc(L);
        for (l = 0; l < L; ++l) {
            int kind = (int)(rnd() % 4);
            p[l] = kind == 0 ? 1 + rnd() % 600 : kind == 1 ? 4096 * (1 + rnd() % 5) + (rnd() % 11) - 5 : kind == 2 ? 4 * (1 + rnd() % 40) : 10000 + rnd() % 300000;
            tb[l] = urand() * 2.0;
            merged[l] = l ? (uint8_t)(rnd() & 1) : 0;
        }
        double a = urand() * 2.0, b = urand() * 2e-6;
        int mode = (int)(rnd() % 4);
        mgwfbp_plan_t *pl = NULL;
        int rc = (rnd() & 1) ? mgwfbp_plan(L, p, tb, urand(), a, b, N, mode, &pl)
                             : mgwfbp_plan_explicit(L, p, tb, urand(), a, b, N, merged, &pl);
        if (rc != MGWFBP_OK) { printf("plan rc %d %s\n", rc, mgwfbp_last_error()); bad++; goto next; }
        {
            static const int tiles[4] = {1024, 2048, 4096, 8192};
            static const int smalls[7] = {0, 1, 64, 512, 1024, 4096, 8192};
            int32_t ng = 0, *gol = malloc(sizeof(int32_t) * L);
            uint64_t *off = malloc(sizeof(uint64_t) * L), ns = 0, nt = 0;
            double t1, t2;
            mgwfbp_plan_set_option(pl, MGWFBP_OPT_TILE_ELEMS, tiles[rnd() % 4]);
            mgwfbp_plan_set_option(pl, MGWFBP_OPT_SMALL_ELEMS, smalls[rnd() % 7]);
            mgwfbp_plan_set_option(pl, MGWFBP_OPT_LONG_TILES, (int)(rnd() % 3) - 1);
            mgwfbp_plan_set_option(pl, MGWFBP_OPT_PAD_ELEMS, (rnd() & 1) ? 4 : 0);
            mgwfbp_plan_info(pl, &ng, gol, off, NULL, &t1, &t2);
            uint64_t *ge = malloc(sizeof(uint64_t) * ng);
            double *mu = malloc(sizeof(double) * L), *gs = malloc(sizeof(double) * ng), *gf = malloc(sizeof(double) * ng);
            mgwfbp_plan_info(pl, NULL, NULL, NULL, ge, NULL, NULL);
            mgwfbp_plan_timeline(pl, mu, gs, gf);
            if (mgwfbp_plan_layout(pl, &ns, NULL, 0, &nt, NULL, 0) != MGWFBP_OK) bad++;
            uint64_t *segs = malloc(sizeof(uint64_t) * MGWFBP_LAYOUT_SEGMENT_COLS * (ns ? ns : 1)), *tl = malloc(sizeof(uint64_t) * MGWFBP_LAYOUT_TILE_COLS * (nt ? nt : 1));
            if (mgwfbp_plan_layout(pl, NULL, segs, ns, NULL, tl, nt) != MGWFBP_OK) bad++;
            if (nt > 1 && mgwfbp_plan_layout(pl, NULL, NULL, 0, NULL, tl, nt - 1) != MGWFBP_EINVAL) bad++;
            size_t wsb = 0;
            mgwfbp_workspace_bytes(pl, -1, &wsb);
            mgwfbp_workspace_bytes(pl, ng - 1, &wsb);
            if (mgwfbp_workspace_bytes(pl, ng, &wsb) == MGWFBP_OK) bad++;
            /* launches on an unbound plan must be refused, not crash */
            if (mgwfbp_pack_reduce_unpack(pl, -1, NULL, 0, NULL) != MGWFBP_ESTATE) bad++;
            if (mgwfbp_step(pl, 0, 0.1f, 0.9f, NULL, 0, NULL) != MGWFBP_ESTATE) bad++;
            if (mgwfbp_tune(pl, NULL, NULL, NULL) != MGWFBP_ESTATE) bad++;
            {
                int32_t flag = 0;
                double t_it = 0.0;
                int dummy_a = 0, dummy_b = 0;   /* two different stream handles; nothing is launched */
                if (mgwfbp_gated_launch(pl, 0, 0.0f, 0.0f, 1u, 10.0, NULL) != MGWFBP_ESTATE) bad++;
                if (mgwfbp_gated_signal(pl, 0, 1u, NULL) != MGWFBP_ESTATE) bad++;
                if (mgwfbp_gated_gave_up(pl, &flag) != MGWFBP_ESTATE) bad++;
                if (mgwfbp_streams_side_by_side(pl, &dummy_a, &dummy_b, &flag) != MGWFBP_ESTATE) bad++;
                if (mgwfbp_run_iteration_gated(pl, NULL, 0, 0.0f, 0.0f, &dummy_a, &dummy_b, 10.0, &t_it) != MGWFBP_ESTATE) bad++;
                if (mgwfbp_plan_set_option(pl, MGWFBP_OPT_GATED_WGS_PER_CU, 16) != MGWFBP_EINVAL) bad++;
                if (mgwfbp_plan_set_option(pl, MGWFBP_OPT_GATED_CUS, -1) != MGWFBP_EINVAL) bad++;
                if (mgwfbp_plan_set_option(pl, MGWFBP_OPT_GATED_CUS, (int)(rnd() % 9) * 32) != MGWFBP_OK) bad++;
                if (mgwfbp_gated_workgroups(pl, 0, NULL, NULL) != MGWFBP_ESTATE) bad++;
                if (mgwfbp_confined_stream_create(128, NULL) != MGWFBP_EINVAL) bad++;
                if (mgwfbp_confined_stream_destroy(NULL) != MGWFBP_OK) bad++;
                if (mgwfbp_plan_set_option(pl, MGWFBP_OPT_GATED_WGS_PER_CU, (int)(rnd() % 15) + 1) != MGWFBP_OK) bad++;
            }
            free(gol); free(off); free(ge); free(mu); free(gs); free(gf); free(segs); free(tl);
        }
        {
            int32_t nw[5] = {4, 8, 16, 32, 64};
            double ti[5], sp[5];
            if (mgwfbp_scaling_curve(L, p, tb, 1.0, (int)(rnd() % 4), 0.045, 8e-7, 1e-9, 5, nw, mode, ti, sp) != MGWFBP_OK) bad++;
        }
        mgwfbp_plan_destroy(pl);
    next:
        free(p); free(tb); free(merged);
    }
    {
        double x[50], y[50], a, b; int i;
        for (i = 0; i < 50; ++i) { x[i] = 1000.0 * (i + 1); y[i] = 0.01 + 1e-6 * x[i] + 1e-4 * urand(); }
        if (mgwfbp_fit_cost(50, x, y, &a, &b) != MGWFBP_OK) bad++;
        if (mgwfbp_fit_cost(1, x, y, &a, &b) == MGWFBP_OK) bad++;
    }
    printf("done, bad = %d\n", bad);
    return bad != 0;
}
