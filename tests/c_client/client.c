/* A plain C99 client of include/jacobi.h: proves that the header is valid C, that the library links
 * from C, and exercises the calls that touch no device (plan creation, layout, options, pass planning,
 * argument errors).  Built and run by tests/test_abi.py; prints one line per check it made. */
#include <stdio.h>
#include <string.h>
#include "jacobi.h"

#define CHECK(cond)                                                 \
    do {                                                            \
        if (!(cond)) {                                              \
            printf("FAILED line %d: %s\n", __LINE__, #cond);        \
            return 1;                                               \
        }                                                           \
    } while (0)

int main(void)
{
    const int64_t dims[2] = {4096, 4096}, tiles[2] = {4, 4}, bad_tiles[2] = {4, 5};
    jacobi_plan *plan = NULL;
    jacobi_layout lay;
    int depths[64], npasses = 0;
    int64_t v = -1;

    CHECK(jacobi_create(&plan, 2, dims, bad_tiles, JACOBI_F64) == JACOBI_ENOTDIV && plan == NULL);
    CHECK(strlen(jacobi_last_error()) > 0);
    CHECK(jacobi_create(&plan, 4, dims, tiles, JACOBI_F64) == JACOBI_EINVAL);
    CHECK(jacobi_create(&plan, 2, dims, tiles, JACOBI_F64) == JACOBI_OK && plan != NULL);
    CHECK(jacobi_get_layout(plan, &lay) == JACOBI_OK);
    CHECK(lay.ndim == 2 && lay.ntiles == 16 && lay.tile[1] == 1024 && lay.tile[2] == 1024);
    CHECK((size_t)lay.grid_bytes == jacobi_grid_bytes(plan));
    CHECK(jacobi_scratch_bytes(plan) >= 16);
    CHECK(jacobi_set_option(plan, "tblock", 8) == JACOBI_OK);
    CHECK(jacobi_get_option(plan, "tblock", &v) == JACOBI_OK && v == 8);
    CHECK(jacobi_set_option(plan, "tblock", 99) == JACOBI_EINVAL);
    CHECK(jacobi_set_option(plan, "no_such_option", 1) == JACOBI_EINVAL);
    CHECK(jacobi_pass_schedule(plan, 20, depths, 64, &npasses) == JACOBI_OK);
    CHECK(npasses == 3 && depths[0] + depths[1] + depths[2] == 20 && depths[0] <= 8);      /* 7 + 7 + 6 */
    /* argument errors are reported before any device call */
    CHECK(jacobi_sweep(plan, NULL, NULL, 1, NULL, NULL) == JACOBI_EINVAL);
    CHECK(jacobi_run(plan, NULL, NULL, 10, 5, NULL, NULL, NULL) == JACOBI_EINVAL);
    CHECK(residual_norm(plan, NULL, NULL, NULL) == JACOBI_EINVAL);
    CHECK(residual_norm_noalloc(plan, NULL, NULL, NULL) == JACOBI_EINVAL);
    CHECK(halo_exchange(NULL, NULL, NULL) == JACOBI_EINVAL);
    CHECK(jacobi_destroy(plan) == JACOBI_OK);
    CHECK(jacobi_destroy(NULL) == JACOBI_OK);
    printf("c client ok\n");
    return 0;
}
