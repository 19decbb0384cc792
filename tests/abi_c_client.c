/* A plain C99 client of the C ABI: built and run by tests/test_abi_cpu.py without a GPU.  It shows
 * that include/aes_spmm.h compiles as C, that the shared library links from C with nothing but the
 * header, and that argument errors come back as status codes with a message (no launch is reached). */
#include <stdio.h>
#include <string.h>

#include "aes_spmm.h"

#define CHECK(cond)                                                       \
    do {                                                                  \
        if (!(cond)) {                                                    \
            printf("FAILED line %d: %s\n", __LINE__, #cond);              \
            return 1;                                                     \
        }                                                                 \
    } while (0)

int main(void)
{
    float dummy[4] = {0};
    int64_t row[2] = {0, 0};
    void *fake = dummy;                       /* never dereferenced: the checks below fail first */

    CHECK(aes_sample_capacity(10, 100, 4) == 40);
    CHECK(aes_sample_capacity(10, 100, 0) == 100);
    CHECK(aes_sample_workspace_bytes(0) == 8);
    CHECK(aes_quantize_workspace_bytes(1000, 128, AES_Q_PER_ROW) == 0);
    CHECK(aes_quantize_workspace_bytes(1000, 128, AES_Q_PER_COLUMN) > 0);

    CHECK(aes_spmm_f32(-1, 4, 0, row, fake, fake, NULL, fake, 8, 8, fake, 8, NULL) == AES_ERR_INVALID_ARG);
    CHECK(strstr(aes_last_error(), "aes_spmm_f32") != NULL);
    CHECK(aes_spmm_f32(4, 4, 0, row, fake, fake, NULL, fake, 4, 8, fake, 8, NULL) == AES_ERR_INVALID_ARG);
    CHECK(aes_spmm_f32(0, 4, 0, row, fake, fake, NULL, fake, 8, 8, NULL, 8, NULL) == AES_OK);
    CHECK(aes_sample_build(4, 4, 8, row, fake, fake, 4, 0, AES_STRATEGY_ADAPTIVE, row, fake, fake, NULL, NULL, NULL, 0,
                           NULL) == AES_ERR_WORKSPACE);
    CHECK(strstr(aes_last_error(), "workspace") != NULL);
    CHECK(aes_quantize_features(4, 8, fake, 8, 7, AES_Q_PER_ROW, fake, 8, fake, fake, NULL, 0, NULL) ==
          AES_ERR_INVALID_ARG);
    CHECK(aes_gcn_layer_f32(4, 4, 0, row, fake, fake, fake, 8, 8, fake, 4, 8, fake, 8, NULL) == AES_ERR_INVALID_ARG);
    CHECK(aes_sample_build_noalloc((int64_t)AES_NOALLOC_MAX_ROWS + 1, 4, 8, row, fake, fake, 4, 0, AES_STRATEGY_ADAPTIVE, row,
                                   fake, fake, NULL, NULL, NULL) == AES_ERR_UNSUPPORTED);
    printf("abi c client ok\n");
    return 0;
}
