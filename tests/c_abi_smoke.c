/* Plain C99 client of include/checkfree.h: no C++, no PyTorch.  Proves the
 * boundary is a C ABI and exercises it end to end with closed-form inputs.
 *
 *   c_abi_smoke --host-only   host-only entry points (no device needed)
 *   c_abi_smoke               also the device path, on HIP device 0
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "checkfree.h"

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            fprintf(stderr, "FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond); \
            return 1;                                                      \
        }                                                                  \
    } while (0)

static int host_only(void)
{
    cf_tuning t;
    cf_tensor d[2];
    uint32_t ct[8], cl[8];
    uint64_t cfirst[8];
    cf_default_tuning(&t);
    CHECK(t.chunk_bytes == 131072u);
    CHECK(strcmp(cf_status_string(CF_OK), "CF_OK") == 0);
    CHECK(cf_recovered_learning_rate(1.0) == 1.1);
    memset(d, 0, sizeof d);
    d[0].data = (void *)0x1000; d[0].numel = 3000; d[0].dtype = CF_F32;
    d[1].data = (void *)0x9000; d[1].numel = 3000; d[1].dtype = CF_F32;
    CHECK(cf_plan_num_chunks(d, 1, 4096) == 3);
    CHECK(cf_plan_chunks(d, 1, 4096, ct, cfirst, cl, 8) == CF_OK);
    CHECK(cfirst[2] == 2048 && cl[2] == 3000 - 2048 && ct[2] == 0);
    CHECK(cf_check_stage_pair(&d[0], 1, &d[1], 1) == CF_OK);
    d[1].data = (void *)0x1004;
    CHECK(cf_check_stage_pair(&d[0], 1, &d[1], 1) == CF_ERR_ALIAS);
    CHECK(cf_ctx_create(0, NULL, NULL) == CF_ERR_NULL);
    CHECK(cf_workspace_bytes() >= 8);
    CHECK(cf_stage_table_bytes(NULL, d, 1) == UINT64_MAX);
    CHECK(cf_ctx_create_in(0, NULL, NULL, 256, NULL, NULL) == CF_ERR_NULL);
    {
        /* an 8-stage pipeline loses its first stage and stage 4 */
        const uint32_t lost[2] = {0, 4};
        cf_recovery_step steps[2];
        uint32_t order[8];
        CHECK(cf_plan_recovery(8, lost, 2, 0, steps) == CF_ERR_VALUE);     /* CheckFree alone cannot rebuild an end stage */
        CHECK(cf_plan_recovery(8, lost, 2, 1, steps) == CF_OK);
        CHECK(steps[0].kind == CF_RECOVER_COPY && steps[0].prev == 1 && steps[0].next == 1);
        CHECK(steps[1].kind == CF_RECOVER_WEIGHTED_AVG && steps[1].prev == 3 && steps[1].next == 5);
        CHECK(cf_plus_stage_order(8, 3, order) == CF_OK);
        CHECK(order[0] == 1 && order[1] == 0 && order[2] == 2 && order[6] == 7 && order[7] == 6);
        CHECK(cf_plus_stage_order(8, 4, order) == CF_OK && order[0] == 0 && order[7] == 7);
    }
    return 0;
}

static int device_path(void)
{
    const uint64_t n = 300007;          /* odd size: several chunks and a ragged tail */
    const float ca = 0.5f, cb = -0.25f, cg = 0.0078125f;   /* 2^-7 */
    float *h = (float *)malloc(n * sizeof(float));
    float *d_a, *d_b, *d_o, *d_g;
    double *d_omega, omega[2];
    cf_ctx *ctx = NULL;
    void *d_ws = NULL, *d_tab_a = NULL, *d_tab_g = NULL;
    uint64_t tab_bytes;
    hipStream_t stream;
    cf_stage *sa = NULL, *sb = NULL, *so = NULL, *sg = NULL;
    const cf_stage *grads[2];
    cf_tensor t;
    uint32_t flags = 7;
    uint64_t k;
    CHECK(h != NULL);
    CHECK(hipMalloc((void **)&d_a, n * 4) == hipSuccess && hipMalloc((void **)&d_b, n * 4) == hipSuccess);
    CHECK(hipMalloc((void **)&d_o, n * 4) == hipSuccess && hipMalloc((void **)&d_g, n * 4) == hipSuccess);
    CHECK(hipMalloc((void **)&d_omega, 2 * sizeof(double)) == hipSuccess);
    for (k = 0; k < n; ++k) h[k] = ca;
    CHECK(hipMemcpy(d_a, h, n * 4, hipMemcpyHostToDevice) == hipSuccess);
    for (k = 0; k < n; ++k) h[k] = cb;
    CHECK(hipMemcpy(d_b, h, n * 4, hipMemcpyHostToDevice) == hipSuccess);
    for (k = 0; k < n; ++k) h[k] = cg;
    CHECK(hipMemcpy(d_g, h, n * 4, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemset(d_o, 0xFF, n * 4) == hipSuccess);

    /* the context and two of the stages in memory this program allocates, set up on its own
     * stream without a wait; the other two stages through the allocating convenience calls */
    CHECK(hipStreamCreateWithFlags(&stream, hipStreamNonBlocking) == hipSuccess);
    CHECK(hipMalloc(&d_ws, cf_workspace_bytes()) == hipSuccess);
    CHECK(cf_ctx_create_in(0, NULL, d_ws, cf_workspace_bytes(), stream, &ctx) == CF_OK);
    memset(&t, 0, sizeof t);
    t.numel = n; t.dtype = CF_F32;
    t.data = d_a;
    tab_bytes = cf_stage_table_bytes(ctx, &t, 1);
    CHECK(tab_bytes != UINT64_MAX && tab_bytes > 0);
    CHECK(hipMalloc(&d_tab_a, tab_bytes) == hipSuccess && hipMalloc(&d_tab_g, tab_bytes) == hipSuccess);
    CHECK(cf_stage_create_in(ctx, &t, 1, d_tab_a, tab_bytes - 1, stream, &sa) == CF_ERR_LIMIT);
    CHECK(cf_stage_create_in(ctx, &t, 1, d_tab_a, tab_bytes, stream, &sa) == CF_OK);
    t.data = d_g; CHECK(cf_stage_create_in(ctx, &t, 1, d_tab_g, tab_bytes, stream, &sg) == CF_OK);
    CHECK(hipStreamSynchronize(stream) == hipSuccess);     /* the calls below use the default stream */
    t.data = d_b; CHECK(cf_stage_create(ctx, &t, 1, &sb) == CF_OK);
    t.data = d_o; CHECK(cf_stage_create(ctx, &t, 1, &so) == CF_OK);
    CHECK(cf_stage_numel(sa) == n && cf_stage_nbytes(sa) == 4 * n && cf_stage_num_tensors(sa) == 1);

    /* omega of the constant gradient, and of the (constant) stage b used as a second "gradient" */
    grads[0] = sg; grads[1] = sb;
    CHECK(cf_stage_grad_sqnorm(ctx, grads, 2, d_omega, NULL) == CF_OK);
    CHECK(hipMemcpy(omega, d_omega, sizeof omega, hipMemcpyDeviceToHost) == hipSuccess);
    CHECK(omega[0] == (double)n * cg * cg);          /* exact: all partial sums are dyadic */
    CHECK(omega[1] == (double)n * cb * cb);

    /* weighted average of two constant stages with the omegas just computed (device pointers) */
    CHECK(cf_recover_stage_weighted_avg(ctx, sa, sb, d_omega, d_omega + 1, so, NULL) == CF_OK);
    CHECK(hipMemcpy(h, d_o, n * 4, hipMemcpyDeviceToHost) == hipSuccess);
    {
        const double want = (omega[0] * ca + omega[1] * cb) / (omega[0] + omega[1]);
        for (k = 0; k < n; ++k) CHECK(h[k] == (float)want);
    }
    /* host weights: 3:1 between 0.5 and -0.25 is 0.3125 exactly */
    CHECK(cf_recover_stage_with_weights(ctx, sa, sb, 3.0, 1.0, so, NULL) == CF_OK);
    CHECK(hipMemcpy(h, d_o, n * 4, hipMemcpyDeviceToHost) == hipSuccess);
    for (k = 0; k < n; ++k) CHECK(h[k] == 0.3125f);
    /* CheckFree+ copy */
    CHECK(cf_copy_stage(ctx, sg, so, NULL) == CF_OK);
    CHECK(hipMemcpy(h, d_o, n * 4, hipMemcpyDeviceToHost) == hipSuccess);
    for (k = 0; k < n; ++k) CHECK(h[k] == cg);
    /* a replica refresh in two slices */
    CHECK(hipMemset(d_o, 0, n * 4) == hipSuccess);
    CHECK(cf_stage_num_chunks(so) == 10);                   /* 300007 floats in chunks of 32768 */
    CHECK(cf_copy_stage_range(ctx, sa, so, 0, 4, NULL) == CF_OK);
    CHECK(hipMemcpy(h, d_o, n * 4, hipMemcpyDeviceToHost) == hipSuccess);
    for (k = 0; k < n; ++k) CHECK(h[k] == (k < 4 * 32768 ? ca : 0.0f));
    CHECK(cf_copy_stage_range(ctx, sa, so, 4, 6, NULL) == CF_OK);
    CHECK(hipMemcpy(h, d_o, n * 4, hipMemcpyDeviceToHost) == hipSuccess);
    for (k = 0; k < n; ++k) CHECK(h[k] == ca);
    CHECK(cf_copy_stage_range(ctx, sa, so, 9, 2, NULL) == CF_ERR_LIMIT);
    CHECK(cf_read_flags(ctx, NULL, &flags, 0) == CF_OK && flags == 0);
    /* errors */
    CHECK(cf_ctx_destroy(ctx) == CF_ERR_CONTEXT);    /* stages alive */
    CHECK(cf_stage_destroy(sa) == CF_OK && cf_stage_destroy(sb) == CF_OK);
    CHECK(cf_stage_destroy(so) == CF_OK && cf_stage_destroy(sg) == CF_OK);
    CHECK(cf_ctx_destroy(ctx) == CF_OK);
    CHECK(hipStreamDestroy(stream) == hipSuccess);
    hipFree(d_ws); hipFree(d_tab_a); hipFree(d_tab_g);
    hipFree(d_a); hipFree(d_b); hipFree(d_o); hipFree(d_g); hipFree(d_omega);
    free(h);
    return 0;
}

int main(int argc, char **argv)
{
    if (host_only()) return 1;
    if (argc > 1 && strcmp(argv[1], "--host-only") == 0) {
        printf("c_abi_smoke: host-only ok\n");
        return 0;
    }
    if (device_path()) return 1;
    printf("c_abi_smoke: ok\n");
    return 0;
}
