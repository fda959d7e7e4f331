/* Plain-C consumer of include/tgemm.h: proves the header is valid C, that every entry point
 * links, and that argument errors are reported without a GPU.  Built and run by
 * tests/test_abi_host.py with gcc -std=c99 (no HIP headers involved). */
#include <stdio.h>
#include <string.h>

#include "tgemm.h"

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            fprintf(stderr, "abi_check: failed: %s (line %d)\n", #cond, __LINE__); \
            return 1;                                                      \
        }                                                                  \
    } while (0)

int main(void)
{
    float *fake = (float *)(size_t)0x1000; /* never dereferenced: every call below is rejected or empty */
    char buf[128];

    CHECK(tg_version() >= 100);
    CHECK(strcmp(tg_status_string(TG_OK), "TG_OK") == 0);
    CHECK(tg_sgemm(-1, 1, 1, fake, 1, fake, 1, fake, 1, NULL) == TG_ERR_INVALID_ARG);
    CHECK(strstr(tg_last_error(), "negative") != NULL);
    CHECK(tg_sgemm(0, 8, 8, NULL, 8, NULL, 8, NULL, 8, NULL) == TG_OK);
    CHECK(tg_sgemm_splitk_static(-1, 1, 1, fake, 1, fake, 1, fake, 1, NULL) == TG_ERR_INVALID_ARG);
    CHECK(tg_sgemm_splitk_static(0, 8, 8, NULL, 8, NULL, 8, NULL, 8, NULL) == TG_OK);
    /* 2 * m * n * 4 bytes beyond the static scratch: refused before any GPU call */
    CHECK(tg_sgemm_splitk_static(4096, 4096, 4096, fake, 4096, fake, 4096, fake, 4096, NULL) == TG_ERR_WORKSPACE);
    CHECK(strstr(tg_last_error(), "static scratch") != NULL);
    CHECK(TG_STATIC_SCRATCH_BYTES == 32u * 1024 * 1024);
    CHECK(tg_sgemm_batched(2, 4, 4, 4, fake, 4, 16, fake, 4, 16, fake, 4, 8, NULL) == TG_ERR_INVALID_ARG);
    CHECK(tg_sgemm_strided(4, 4, 4, fake, 4, 0, fake, 4, 1, fake, 4, NULL) == TG_ERR_INVALID_ARG);
    CHECK(tg_saxpy(-5, 1.0f, fake, fake, fake, NULL) == TG_ERR_INVALID_ARG);
    CHECK(tg_saxpy(0, 1.0f, NULL, NULL, NULL, NULL) == TG_OK);
    CHECK(tg_tune(1, 4, 4, 8, fake, 7, 0, fake, 4, 0, fake, 4, 0, NULL, 3) == TG_ERR_INVALID_ARG);
    CHECK(tg_set_workspace(NULL, 16) == TG_ERR_INVALID_ARG);
    CHECK(tg_set_workspace(NULL, 0) == TG_OK);
    CHECK(tg_workspace_bytes(1, 1024, 1024, 1024) > 0);
    CHECK(tg_strided_workspace_bytes(1024, 1024, 1024, 32, 1) >= tg_workspace_bytes(1, 1024, 1024, 1024) + 4u * 1024 * 1024);
    CHECK(tg_strided_workspace_bytes(1024, 1024, 1024, 0, 1) == 0);
    CHECK(tg_tune_is_launch_bound(1, 256, 256, 32) == 1 && tg_tune_is_launch_bound(1, 4096, 4096, 4096) == 0);
    CHECK(tg_tune_is_launch_bound(1, 0, 4, 4) == -1);
    CHECK(tg_num_kernels() > 0);
    CHECK(tg_kernel_name(0, buf, sizeof buf) == TG_OK && strlen(buf) > 0);
    CHECK(tg_force_config("no_such_kernel") == TG_ERR_INVALID_ARG);
    CHECK(tg_force_config(NULL) == TG_OK);
    CHECK(tg_get_config(1, 4096, 4096, 4096, buf, sizeof buf) == TG_OK && strstr(buf, "acc2") != NULL);
    CHECK(tg_last_config() != NULL);
    CHECK(tg_get_math() == TG_MATH_FP32_MFMA && tg_set_math(99) == TG_ERR_INVALID_ARG);
    CHECK(tg_set_math(TG_MATH_BF16_PIECES) == TG_OK && tg_get_math() == TG_MATH_BF16_PIECES);
    CHECK(tg_get_config(1, 4096, 4096, 4096, buf, sizeof buf) == TG_OK && buf[0] == 'e');
    CHECK(tg_set_math(TG_MATH_FP32_MFMA) == TG_OK);
    {
        double bound = 0, model = 0;
        CHECK(tg_num_candidates(1, 4096, 4096, 4096) > 0);
        CHECK(tg_candidate(1, 4096, 4096, 4096, 0, buf, sizeof buf, &bound, &model) == TG_OK);
        CHECK(bound > 800.0 && model >= bound && strstr(buf, "acc2") != NULL);
        CHECK(tg_candidate(1, 4096, 4096, 4096, -1, buf, sizeof buf, NULL, NULL) == TG_ERR_INVALID_ARG);
    }
    CHECK(tg_load_tune_cache("/nonexistent/file") == TG_ERR_INVALID_ARG);
    tg_clear_tune_cache();
    printf("abi_check: ok (%d kernel variants, version %d)\n", tg_num_kernels(), tg_version());
    return 0;
}
