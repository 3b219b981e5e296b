/* The boundary from plain C99, with no Python in between: a host-only plan is built,
 * queried, saved, loaded and destroyed, and bad arguments come back as error codes with a
 * message.  Compiled and run by tests/test_abi_and_plan.py. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "sparsert.h"

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "line %d: %s (%s)\n", __LINE__, #cond, sparsert_last_error()); return 1; } } while (0)

int main(void)
{
    /* 3 x 4 matrix: rows {0:1.0, 2:-2.0}, {}, {1:0.5, 2:4.0, 3:8.0} */
    const int32_t row_ptr[4] = {0, 2, 2, 5};
    const int32_t col_idx[5] = {0, 2, 1, 2, 3};
    const float vals[5] = {1.0f, -2.0f, 0.5f, 4.0f, 8.0f};
    sparsert_options opt;
    sparsert_plan *plan = NULL, *again = NULL;
    int32_t info[SPARSERT_INFO_COUNT], perm[3];
    size_t need = 0;
    void *blob;

    memset(&opt, 0, sizeof(opt));
    opt.host_only = 1;
    opt.kernel = SPARSERT_KERNEL_SPEC;
    opt.spec_rows = 2;
    CHECK(sparsert_version() >= 100);
    CHECK(sparsert_inspect(row_ptr, col_idx, vals, 3, 4, 70, &opt, &plan) == SPARSERT_OK && plan);
    CHECK(sparsert_plan_export(plan, SPARSERT_FIELD_INFO, info, sizeof(info), &need) == SPARSERT_OK && need == sizeof(info));
    CHECK(info[SPARSERT_INFO_M] == 3 && info[SPARSERT_INFO_NNZ] == 5 && info[SPARSERT_INFO_KERNEL] == SPARSERT_KERNEL_SPEC);
    CHECK(info[SPARSERT_INFO_SPEC_CODE_BYTES] > 0 && info[SPARSERT_INFO_SPEC_GROUPS] == 2);
    CHECK(sparsert_plan_export(plan, SPARSERT_FIELD_PERM, perm, sizeof(perm), NULL) == SPARSERT_OK);
    CHECK(perm[0] == 2 && perm[1] == 0 && perm[2] == 1);   /* rows by nonzero count, descending */

    CHECK(sparsert_plan_save(plan, NULL, 0, &need) == SPARSERT_OK && need > 24);
    blob = malloc(need);
    CHECK(blob != NULL);
    CHECK(sparsert_plan_save(plan, blob, need, NULL) == SPARSERT_OK);
    CHECK(sparsert_plan_load(blob, need, 1, &again) == SPARSERT_OK && again);
    CHECK(sparsert_plan_export(again, SPARSERT_FIELD_PERM, perm, sizeof(perm), NULL) == SPARSERT_OK && perm[0] == 2);
    CHECK(sparsert_plan_load(blob, need - 1, 1, &again) == SPARSERT_EINVAL && again == NULL);
    free(blob);

    /* a host-only plan cannot be executed; errors carry a message */
    CHECK(sparsert_spmm(plan, (const void *)16, (void *)32, NULL) == SPARSERT_EINVAL);
    CHECK(strlen(sparsert_last_error()) > 0);
    CHECK(sparsert_inspect(row_ptr, col_idx, vals, 3, 2, 70, &opt, &again) == SPARSERT_EINVAL);   /* column 3 >= K */
    sparsert_plan_destroy(plan);
    sparsert_plan_destroy(NULL);
    puts("c abi ok");
    return 0;
}
