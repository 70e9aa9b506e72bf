/* A plain C client of the library's ABI: includes both headers as C, calls what can be called without a GPU (version,
 * error strings, the host-side selection rules, argument validation).  Built and run by tests/test_c_abi_client.py. */
#include <stdio.h>
#include <string.h>

#include "gemm_f32.h"
#include "gemm_f64.h"

int main(void)
{
    int variant = -1, splits = -1, chunk = -1;
    int64_t tm = -1, tn = -1;
    double fake[4];
    if (gemm_f64_version() < 300) return 1;
    if (strcmp(gemm_f64_strerror(GEMM_F64_OK), "success") != 0) return 2;
    if (gemm_f64_variant_count() != gemm_f32_variant_count() || gemm_f64_variant_name(0) == NULL) return 3;
    if (gemm_f64_choose_variant(8192, 8192, 8192, 256) < 1) return 4;
    if (gemm_f64_choose_variant_general(1, 1, 300, 300, 300, 256) < 1) return 5;
    if (gemm_f64_tile_of_block(5, 4, 4, &tm, &tn) != GEMM_F64_OK || tm < 0 || tm > 3 || tn < 0 || tn > 3) return 6;
    if (gemm_f64_split_k_plan(0, 0, 640, 640, 8192, 256, (int64_t)1 << 40, &variant, &splits, &chunk) != GEMM_F64_OK || splits < 2)
        return 7;
    if (gemm_f64_split_k_workspace_bytes(0, 0, 640, 640, 8192, 256) != (int64_t)splits * 640 * 640 * 8) return 8;
    /* rejected before anything touches a device */
    if (gemm_f64(-1, 2, 2, fake, 2, fake, 2, fake, 2, NULL) != GEMM_F64_ERR_DIM) return 9;
    if (gemm_f64_general(0, 0, 2, 2, 3, 1.0, fake, 2, fake, 2, 1.0, fake, 2, NULL) != GEMM_F64_ERR_LDA) return 10;
    if (gemm_f32_general(0, 3, 2, 2, 2, 1.0f, (const float *)fake, 2, (const float *)fake, 2, 1.0f, (float *)fake, 2, NULL) != GEMM_F64_ERR_DIM)
        return 11;
    if (gemm_f64_general_ws(0, 0, 0, 2, 2, 1.0, NULL, 2, NULL, 2, 1.0, NULL, 2, NULL, 8, NULL) != GEMM_F64_ERR_NULL) return 12;
    if (gemm_f64_strided(2, 3, 4, 1.0, fake, 4, 1, fake, 3, 1, 1.0, fake, 2, 1, NULL) != GEMM_F64_ERR_LDC) return 13;
    if (gemm_f32_strided(2, 3, 4, 0.0f, NULL, 1, 2, NULL, 1, 4, 1.0f, (float *)fake, 1, 2, NULL) != GEMM_F64_OK) return 14;
    puts("c abi client ok");
    return 0;
}
