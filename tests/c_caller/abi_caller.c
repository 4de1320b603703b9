/* A C caller of the lnpegn library: includes only the public header, links against
 * liblnpegn.so, and exercises entry points that do their work (or fail validation) on the
 * host, so it runs on a machine without a GPU.  Prints one line per check; exit 0 = all ok. */
#include <stdio.h>
#include <string.h>

#include "lnpegn.h"

static int failures = 0;
#define CHECK(cond)                                                     \
    do {                                                                \
        if (!(cond)) {                                                  \
            printf("FAIL line %d: %s\n", __LINE__, #cond);              \
            ++failures;                                                 \
        }                                                               \
    } while (0)

int main(void)
{
    /* fake, never dereferenced: every call below is rejected before a launch */
    void *x = (void *)0x1000, *dy = (void *)0x2000, *gamma = (void *)0x3000, *dx = (void *)0x4000;
    float *dgamma = (float *)0x5000, *dbeta = (float *)0x6000;
    void *ws = (void *)0x100000;
    const size_t huge = (size_t)1 << 40;

    const size_t need = lnpegn_workspace_bytes(16, 2048, 2048, LNPEGN_BF16);
    CHECK(need > 0 && need % 256 == 0);
    CHECK(lnpegn_workspace_bytes(0, 1, 1, LNPEGN_F32) == 0);
    CHECK(strcmp(lnpegn_status_string(LNPEGN_OK), "ok") == 0);
    CHECK(strcmp(lnpegn_status_string(LNPEGN_EWORKSPACE), "workspace missing or too small") == 0);
    CHECK(strcmp(lnpegn_status_string(1234), "unknown status") == 0);

    CHECK(gns_linear_accum_steps(0, 800, 8) == 1);
    CHECK(gns_linear_accum_steps(101, 800, 8) == 2);
    CHECK(gns_linear_accum_steps(800, 800, 8) == 8);
    CHECK(gns_linear_accum_steps((int64_t)1 << 62, INT64_MAX, 2147483647) == 1073741824);
    CHECK(gns_linear_accum_steps(-1, 800, 8) == -LNPEGN_EINVAL);

    CHECK(ln_bwd(x, dy, gamma, NULL, NULL, dx, dgamma, dbeta, 0, 3, 8, LNPEGN_BF16, LNPEGN_BF16, 1e-5f, ws, huge,
                 NULL) == LNPEGN_EINVAL);
    CHECK(ln_bwd(NULL, dy, gamma, NULL, NULL, dx, dgamma, dbeta, 2, 3, 8, LNPEGN_BF16, LNPEGN_BF16, 1e-5f, ws, huge,
                 NULL) == LNPEGN_EINVAL);
    CHECK(ln_bwd(x, dy, gamma, NULL, NULL, x, dgamma, dbeta, 2, 3, 8, LNPEGN_BF16, LNPEGN_BF16, 1e-5f, ws, huge,
                 NULL) == LNPEGN_EINVAL);
    CHECK(ln_bwd(x, dy, gamma, NULL, NULL, dx, dgamma, dbeta, 2, 3, 8, (lnpegn_dtype)7, LNPEGN_BF16, 1e-5f, ws, huge,
                 NULL) == LNPEGN_EUNSUPPORTED);
    CHECK(ln_bwd(x, dy, gamma, NULL, NULL, dx, dgamma, dbeta, 2, 3, 8, LNPEGN_BF16, LNPEGN_BF16, 1e-5f, NULL, huge,
                 NULL) == LNPEGN_EWORKSPACE);
    CHECK(ln_bwd(x, dy, gamma, NULL, NULL, dx, dgamma, dbeta, 2, 3, 8, LNPEGN_BF16, LNPEGN_BF16, 1e-5f, ws, 16,
                 NULL) == LNPEGN_EWORKSPACE);
    CHECK(ln_bwd(x, dy, gamma, NULL, NULL, dx, dgamma, dbeta, 2, 3, 8, LNPEGN_BF16, LNPEGN_BF16, -1.0f, ws, huge,
                 NULL) == LNPEGN_EINVAL);
    CHECK(gns_estimate((const float *)x, (const float *)dy, 1, 1, 1.0f, (float *)dx, NULL) == LNPEGN_EINVAL);
    CHECK(lnpegn_set_tuning(99, 1) == LNPEGN_EINVAL);
    {
        int64_t plan[LNPEGN_PLAN_FIELDS];
        CHECK(lnpegn_plan_query(16, 2048, 2048, LNPEGN_BF16, 1, 1, plan, LNPEGN_PLAN_FIELDS) == LNPEGN_OK);
        CHECK(plan[0] == 1 && plan[5] == 16 * plan[4] && plan[15] == 2048);
        CHECK((size_t)plan[14] <= lnpegn_workspace_bytes(16, 2048, 2048, LNPEGN_BF16));
        CHECK(lnpegn_plan_query(16, 2048, 0, LNPEGN_BF16, 1, 1, plan, LNPEGN_PLAN_FIELDS) == LNPEGN_EINVAL);
    }

    printf(failures ? "%d check(s) failed\n" : "all checks passed (%d failures)\n", failures);
    return failures ? 1 : 0;
}
