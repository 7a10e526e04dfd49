/* A plain C99 client of the library's host-side calls: proves that include/mgwfbp.h is a C
 * header and that the planner is usable without Python, C++ or a GPU.
 * Reads nothing; prints "key value" lines that the test compares with the CPU oracle.
 * Case: the hand-worked three-layer example (t_f = 0, t_b = 0.9 each, a = 1, b*M = 10 each). */
#include <stdio.h>
#include <string.h>

#include "mgwfbp.h"

static int run(int32_t mode, const char *name)
{
    const uint64_t p[3] = {2500000u, 2500000u, 2500000u}; /* 10^7 bytes each */
    const double tb[3] = {0.9, 0.9, 0.9};
    mgwfbp_plan_t *pl = NULL;
    int32_t n_groups = 0, group_of_layer[3];
    uint64_t off[3], gelems[3];
    double t_iter = 0.0, t_wfbp = 0.0;
    int rc = mgwfbp_plan(3, p, tb, 0.0, 1.0, 1.0e-6, 4, mode, &pl);
    if (rc != MGWFBP_OK) {
        printf("error %d %s\n", rc, mgwfbp_last_error());
        return 1;
    }
    rc = mgwfbp_plan_info(pl, &n_groups, group_of_layer, off, gelems, &t_iter, &t_wfbp);
    if (rc != MGWFBP_OK) return 1;
    printf("%s groups %d t_iter %.17g t_wfbp %.17g layers %d %d %d\n", name, n_groups, t_iter, t_wfbp,
           group_of_layer[0], group_of_layer[1], group_of_layer[2]);
    mgwfbp_plan_destroy(pl);
    return 0;
}

int main(void)
{
    mgwfbp_plan_t *pl = NULL;
    double a = 0.0, b = 0.0;
    if (run(MGWFBP_MODE_OPTIMAL, "optimal") || run(MGWFBP_MODE_PAPER_GREEDY, "theorem1") ||
        run(MGWFBP_MODE_WFBP, "wfbp") || run(MGWFBP_MODE_SINGLE, "single"))
        return 1;
    /* error path: L = 0 must be refused with a message, not crash */
    if (mgwfbp_plan(0, NULL, NULL, 0.0, 1.0, 1.0, 1, MGWFBP_MODE_OPTIMAL, &pl) != MGWFBP_EINVAL) return 2;
    if (strlen(mgwfbp_last_error()) == 0) return 3;
    /* Table II, ring row, 8 workers, alpha = 45.26 us: start-up 2(N-1)alpha */
    if (mgwfbp_table2_cost(3, 8, 0.04526, 8.0e-7, 0.0, &a, &b) != MGWFBP_OK) return 4;
    printf("ring8 a %.17g b %.17g\n", a, b);
    return 0;
}
