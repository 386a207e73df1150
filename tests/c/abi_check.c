/* Plain C99 caller of the library: includes the public header, links against libkmv.so and exercises the
 * entry points that need no device (version, workspace queries, the partition, argument errors, quick returns).
 * Built and run by tests/test_abi.py. */
#include <stdio.h>
#include <string.h>

#include "kmv.h"

#define CHECK(cond)                                              \
    do {                                                         \
        if (!(cond)) {                                           \
            printf("failed: %s (line %d)\n", #cond, __LINE__);   \
            return 1;                                            \
        }                                                        \
    } while (0)

int main(void) {
    const float one = 1.0f, zero = 0.0f;
    float dummy[4] = {0, 0, 0, 0};
    int64_t w = -1, s = -1;
    CHECK(strstr(kmv_version(), "kmv") != NULL);
    CHECK(kmv_gemv_workspace_bytes('d', 'N', 4096, 4096) > 0);
    CHECK(kmv_symv_workspace_bytes('z', 'U', 4096) >= 4096 * sizeof(kmv_complex128));
    CHECK(kmv_gemv_workspace_bytes('q', 'N', 8, 8) == 0);
    kmv_partition(10, 4, 1, &w, &s);
    CHECK(w == 3 && s == 3);                       /* shares 3, 3, 2, 2 of 10 items */
    /* argument errors come back before anything touches a device */
    CHECK(kmv_sgemv('X', 4, 4, &one, dummy, 4, dummy, 1, &zero, dummy, 1, NULL, 0, NULL) == -1);
    CHECK(kmv_sgemv('N', 4, 4, &one, dummy, 3, dummy, 1, &zero, dummy, 1, NULL, 0, NULL) == -6);
    CHECK(kmv_ssymv('L', 4, &one, dummy, 4, dummy, 0, &zero, dummy, 1, NULL, 0, NULL) == -7);
    CHECK(kmv_sgemv('N', 4, 4, NULL, dummy, 4, dummy, 1, &zero, dummy, 1, NULL, 0, NULL) == KMV_ERR_NULL);
    /* quick returns: empty product; alpha = 0 with beta = 1 */
    CHECK(kmv_sgemv('N', 0, 4, &one, dummy, 1, dummy, 1, &zero, dummy, 1, NULL, 0, NULL) == KMV_OK);
    CHECK(kmv_ssymv('U', 4, &zero, NULL, 4, NULL, 1, &one, NULL, 1, NULL, 0, NULL) == KMV_OK);
    CHECK(kmv_set_tuning("no_such_key", 1) == -1 && kmv_get_tuning("wg_target") == 0);
    printf("ok\n");
    return 0;
}
