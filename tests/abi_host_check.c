/* Exercises every host-side path of the C ABI that needs no GPU work: size functions, names, argument
 * checks, call-order checks.  Built and run by tests/test_abi_loads.py against a build of the library
 * whose host code is instrumented with AddressSanitizer and UBSan; prints "ok" and exits 0 if every
 * check holds (a sanitizer report makes the process fail by itself). */
#include <stdio.h>
#include <string.h>

#include "../include/excp.h"

static int fails = 0;
#define CHECK(c) do { if (!(c)) { printf("FAIL line %d: %s\n", __LINE__, #c); ++fails; } } while (0)

int main(void) {
    /* closed-form sizes */
    CHECK(excp_blob_bound(0, 4) == 80 + 3 * 16 * 4);
    CHECK(excp_blob_size(1000, 345, 76, 4) == 80 + 192 + 128 + 48 + 176 + 2 * 48);
    CHECK(excp_blob_size(10, 11, 0, 4) == 0 && excp_blob_bound(10, 9) == 0 && excp_blob_bound(10, 1) == 0);
    CHECK(excp_blob_size_ex(100, 50, 70, 4, EXCP_FLAG_NO_W2M) != 0 && excp_blob_size_ex(100, 50, 70, 4, 0) == 0);
    CHECK(excp_blob_size_ex(100, 50, 20, 32, EXCP_FLAG_NO_QUANT) != 0 && excp_blob_size_ex(100, 50, 20, 4, EXCP_FLAG_NO_QUANT) == 0);
    CHECK(excp_blob_size_ex(1, 1, 1, 4, EXCP_FLAG_W_F16 | EXCP_FLAG_W_BF16) == 0 && excp_blob_size_ex(1, 1, 1, 4, 64u) == 0);
    CHECK(excp_blob_bound(EXCP_MAX_TENSOR_ELEMS, 8) > EXCP_MAX_TENSOR_ELEMS);
    CHECK(excp_dense_bytes(7, 4) == 4 && excp_dense_bytes(7, 5) == 7 && excp_head_bytes(4) == 80 + 192 && excp_head_bytes(9) == 0);
    for (int code = 1; code >= -9; --code) CHECK(excp_strerror(code) != NULL && strlen(excp_strerror(code)) > 1);
    CHECK(excp_stage_count() > 10);
    for (int i = -2; i < excp_stage_count() + 2; ++i) CHECK(excp_stage_name(i) != NULL);

    /* argument checks that enqueue nothing */
    excp_ctx *ctx = (excp_ctx *)0x1;
    CHECK(excp_create(NULL, 0, NULL, 1, 1) == EXCP_E_ARG);
    CHECK(excp_create(&ctx, 0, NULL, 0, 0) == EXCP_E_ARG && ctx == NULL);
    CHECK(excp_create(&ctx, 0, NULL, EXCP_MAX_TENSOR_ELEMS + 1, EXCP_MAX_TENSOR_ELEMS + 1) == EXCP_E_ARG && ctx == NULL);
    CHECK(excp_create(&ctx, 0, NULL, 4096, 1024) == EXCP_E_ARG && ctx == NULL);
    CHECK(excp_create(&ctx, -1, NULL, 4096, 4096) == EXCP_E_HIP && ctx == NULL);
    excp_stats st;
    memset(&st, 0x5a, sizeof st);
    uint64_t nbytes = 12345;
    float x[4] = {0};
    CHECK(excp_compress_step(NULL, x, x, x, x, 4, 5e-5f, 2.f, 4, 10, 0, x, 16, &nbytes, NULL, &st) == EXCP_E_ARG);
    CHECK(nbytes == 12345 && ((unsigned char *)&st)[0] == 0x5a);          /* outputs untouched */
    CHECK(excp_decompress_step(NULL, x, x, 16, 4, x, NULL, NULL, 0) == EXCP_E_ARG);
    CHECK(excp_compress_tensors(NULL, 0, NULL, 5e-5f, 2.f, 4, 10, 0) == EXCP_E_ARG);
    CHECK(excp_decompress_tensors(NULL, 0, NULL) == EXCP_E_ARG);
    CHECK(excp_reconstruct_chain(NULL, 0, NULL) == EXCP_E_ARG);
    CHECK(excp_export_dense(NULL, 0, NULL) == EXCP_E_ARG && excp_decompress_dense(NULL, 0, NULL) == EXCP_E_ARG);
    CHECK(excp_collect(NULL, NULL) == EXCP_E_ARG);
    CHECK(excp_set_profiling(NULL, 1) == EXCP_E_ARG && excp_set_param(NULL, EXCP_PARAM_WIDE_ELEMS, 1) == EXCP_E_ARG);
    CHECK(excp_stage_ms(NULL, 0, NULL, NULL) == EXCP_E_ARG && excp_copy_probe(NULL, x, x, 16) == EXCP_E_ARG);
    CHECK(excp_workspace_bytes(NULL) == 0);
    excp_destroy(NULL);
    /* the entry point without a context: refusals come before anything touches a device */
    CHECK(excp_decompress_step_static(0, NULL, x, x, 16, 4, x, NULL, NULL, 0x30) == EXCP_E_ARG);
    CHECK(excp_decompress_step_static(0, NULL, x, x, 16, 4, x, NULL, NULL, 1) == EXCP_E_ARG);
    CHECK(excp_decompress_step_static(0, NULL, x, x, 16, EXCP_STATIC_MAX_ELEMS + 1, x, NULL, NULL, 0) == EXCP_E_ARG);
    CHECK(excp_decompress_step_static(0, NULL, x, NULL, 16, 4, x, NULL, NULL, 0) == EXCP_E_ARG);
    CHECK(excp_decompress_step_static(0, NULL, x, (char *)x + 4, 16, 4, x, NULL, NULL, 0) == EXCP_E_ARG);
    CHECK(excp_decompress_step_static(-1, NULL, x, x, 16, 4, x, NULL, NULL, 0) == EXCP_E_ARG);
    CHECK(excp_decompress_step_static(1 << 20, NULL, x, x, 16, 4, x, NULL, NULL, 0) == EXCP_E_ARG);

    /* with a device present a context is made, used for its call-order checks and destroyed; without
     * one, creation reports the HIP error and leaves nothing behind */
    int rc = excp_create(&ctx, 0, NULL, 4096, 8192);
    CHECK(rc == EXCP_OK || rc == EXCP_E_HIP);
    if (rc == EXCP_OK) {
        CHECK(ctx != NULL && excp_workspace_bytes(ctx) > 0);
        CHECK(excp_collect(ctx, NULL) == EXCP_E_STATE);
        CHECK(excp_set_param(ctx, 99, 1) == EXCP_E_ARG && excp_set_param(ctx, EXCP_PARAM_WIDE_ELEMS, 0) == EXCP_E_ARG);
        CHECK(excp_set_param(ctx, EXCP_PARAM_CAND_LIST_ELEMS, 4096) == EXCP_OK);
        CHECK(excp_compress_tensors(ctx, 5000, NULL, 5e-5f, 2.f, 4, 10, 0) == EXCP_E_ARG);
        CHECK(excp_compress_tensors(ctx, 0, NULL, 5e-5f, 2.f, 9, 10, 0) == EXCP_E_ARG);
        CHECK(excp_compress_tensors(ctx, 0, NULL, -1.f, 2.f, 4, 10, 0) == EXCP_E_ARG);
        excp_destroy(ctx);
    } else {
        CHECK(ctx == NULL);
    }
    if (fails) return 1;
    printf("ok\n");
    return 0;
}
