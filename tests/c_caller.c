/* A plain C99 caller of the boundary: includes the public header, links the shared library and
 * exercises the calls that need no GPU (sizes, options, status strings, and a dry-run plan of the
 * benchmark's headline shape).  Prints one line per check; exit status 0 when all hold. */
#include <stdio.h>
#include <string.h>

#include "elsa.h"

static int fails = 0;
#define CHECK(cond)                                        \
    do {                                                   \
        if (!(cond)) {                                     \
            printf("FAILED %s:%d %s\n", __FILE__, __LINE__, #cond); \
            ++fails;                                       \
        }                                                  \
    } while (0)

int main(void) {
    int v = -1;
    void *dummy = (void *)(size_t)(1u << 20); /* aligned, never dereferenced in a dry run */

    CHECK(strcmp(elsa_status_string(ELSA_OK), elsa_status_string(ELSA_ERR_INVALID_ARG)) != 0);
    CHECK(elsa_split_kv_workspace_bytes(1, 16, 1024, 64, 4) >= (size_t)16 * 4 * 1024 * (64 + 2) * sizeof(float));
    CHECK(elsa_split_kv_workspace_bytes(0, 16, 1024, 64, 4) == 0);

    CHECK(elsa_set_option(ELSA_OPT_DRY_RUN, 1) == ELSA_OK);
    CHECK(elsa_get_option(ELSA_OPT_DRY_RUN, &v) == ELSA_OK && v == 1);
    CHECK(elsa_set_option(ELSA_OPT_DRY_RUN, 7) == ELSA_ERR_INVALID_ARG);
    CHECK(elsa_set_option(99, 0) == ELSA_ERR_UNSUPPORTED);

    /* headline shape: B = 1, H = 16, n = 16384, d = 64, FP32 */
    CHECK(elsa_attn_fwd(dummy, dummy, dummy, dummy, 1, 16, 16384, 64, 0.125f, 0, ELSA_F32, NULL) == ELSA_OK);
    CHECK(strcmp(elsa_last_kernel(), "mfma_q128_k32") == 0);
    CHECK(elsa_last_splits() == 1);
    /* bad arguments are errors, not launches */
    CHECK(elsa_attn_fwd(NULL, dummy, dummy, dummy, 1, 16, 16384, 64, 0.125f, 0, ELSA_F32, NULL) == ELSA_ERR_INVALID_ARG);
    CHECK(elsa_attn_fwd(dummy, dummy, dummy, dummy, 1, 16, 16384, 48, 0.125f, 0, ELSA_F32, NULL) == ELSA_ERR_UNSUPPORTED);

    CHECK(elsa_set_option(ELSA_OPT_DRY_RUN, 0) == ELSA_OK);
    printf("%s\n", fails ? "c caller: FAILED" : "c caller: ok");
    return fails ? 1 : 0;
}
