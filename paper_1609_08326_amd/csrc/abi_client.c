/*
 * A client of the C ABI in plain C99: no Python, no PyTorch.  Device memory
 * comes from hipMalloc, the library is reached through include/dcasgd.h only.
 * It runs four small cases whose results are known in closed form and prints
 * "abi_client: OK" (exit status 0) if all of them hold:
 *   1. lambda = 0 (the update is ASGD, Eq. 2.2): w = w0 - eta * sum of gradients,
 *      exact for the dyadic values used;
 *   2. Algorithm 2's pull: the returned row equals w bit for bit, other rows stay;
 *   3. DC-ASGD-c with a stale backup, one parameter value worked by hand;
 *   4. the synchronous fold of three gradients, in the caller's order and ranked
 *      by norm - with the caller's workspace and with the library's static one -
 *      each against the value worked by hand.
 */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "dcasgd.h"

#define HIP_OK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    fprintf(stderr, "abi_client: %s: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define DC_OK(x) do { int rc_ = (x); if (rc_ != DCASGD_OK) { \
    fprintf(stderr, "abi_client: %s: %s\n", #x, dcasgd_strerror(rc_)); return 2; } } while (0)

static int all_equal(const float* v, size_t n, float want, const char* what) {
    size_t i;
    for (i = 0; i < n; ++i)
        if (v[i] != want) {
            fprintf(stderr, "abi_client: %s: element %lu is %.9g, expected %.9g\n", what,
                    (unsigned long)i, (double)v[i], (double)want);
            return 0;
        }
    return 1;
}

int main(void) {
    const size_t d = 100003;             /* ragged: not a multiple of four */
    const int M = 3;
    const size_t stride = (d + 63) / 64 * 64;
    float *w = NULL, *bak = NULL, *g = NULL;
    float* host = (float*)malloc(d * sizeof(float));
    const float* row;
    dcasgd_t h;
    size_t i;
    int k;
    if (!host) return 2;
    HIP_OK(hipMalloc((void**)&w, d * sizeof(float)));
    HIP_OK(hipMalloc((void**)&bak, (size_t)M * stride * sizeof(float)));
    HIP_OK(hipMalloc((void**)&g, d * sizeof(float)));

    /* 1. lambda = 0: five pushes of g = 1/4 with eta = 1/2 from w0 = 1 */
    for (i = 0; i < d; ++i) host[i] = 1.0f;
    HIP_OK(hipMemcpy(w, host, d * sizeof(float), hipMemcpyHostToDevice));
    for (i = 0; i < d; ++i) host[i] = 0.25f;
    HIP_OK(hipMemcpy(g, host, d * sizeof(float), hipMemcpyHostToDevice));
    h = dcasgd_create(d, M, 0.5f, 0.0f, DCASGD_MODE_C, 0.0f, 0.0f);
    if (!h) { fprintf(stderr, "abi_client: dcasgd_create failed\n"); return 2; }
    DC_OK(dcasgd_bind(h, w, bak, stride, NULL));
    DC_OK(dcasgd_init(h, NULL));
    for (k = 0; k < 5; ++k) DC_OK(dcasgd_push(h, k % M, g, NULL));
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(host, w, d * sizeof(float), hipMemcpyDeviceToHost));
    if (dcasgd_step(h) != 5 || !all_equal(host, d, 1.0f - 5 * 0.125f, "ASGD case")) return 1;

    /* 2. pull: row 1 becomes w, row 2 still holds w0 */
    row = dcasgd_pull(h, 1);
    if (!row || row != bak + stride) { fprintf(stderr, "abi_client: pull returned a wrong row\n"); return 1; }
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(host, row, d * sizeof(float), hipMemcpyDeviceToHost));
    if (!all_equal(host, d, 0.375f, "pulled row")) return 1;
    HIP_OK(hipMemcpy(host, bak + 2 * stride, d * sizeof(float), hipMemcpyDeviceToHost));
    if (!all_equal(host, d, 1.0f, "untouched row")) return 1;
    DC_OK(dcasgd_destroy(h));

    /* 3. Eq. 4.1 with lambda = 1/4, eta = 1/2: w0 = 2; worker 0 pushes g = 1 (its backup is
     *    w0, so w = 2 - 1/2 = 3/2); worker 1, still at w0, pushes g = 2:
     *    w - w_bak = -1/2, lambda g g = 1, compensated gradient = 2 - 1/2 = 3/2,
     *    w = 3/2 - 3/4 = 3/4. */
    for (i = 0; i < d; ++i) host[i] = 2.0f;
    HIP_OK(hipMemcpy(w, host, d * sizeof(float), hipMemcpyHostToDevice));
    h = dcasgd_create(d, M, 0.5f, 0.25f, DCASGD_MODE_C | DCASGD_PULL_ON_PUSH, 0.0f, 0.0f);
    if (!h) { fprintf(stderr, "abi_client: dcasgd_create failed\n"); return 2; }
    DC_OK(dcasgd_bind(h, w, bak, stride, NULL));
    DC_OK(dcasgd_init(h, NULL));
    for (i = 0; i < d; ++i) host[i] = 1.0f;
    HIP_OK(hipMemcpy(g, host, d * sizeof(float), hipMemcpyHostToDevice));
    DC_OK(dcasgd_push(h, 0, g, NULL));
    HIP_OK(hipDeviceSynchronize());
    for (i = 0; i < d; ++i) host[i] = 2.0f;
    HIP_OK(hipMemcpy(g, host, d * sizeof(float), hipMemcpyHostToDevice));
    DC_OK(dcasgd_push(h, 1, g, NULL));
    HIP_OK(hipDeviceSynchronize());
    HIP_OK(hipMemcpy(host, w, d * sizeof(float), hipMemcpyDeviceToHost));
    if (!all_equal(host, d, 0.75f, "delay-compensated case")) return 1;
    HIP_OK(hipMemcpy(host, bak + stride, d * sizeof(float), hipMemcpyDeviceToHost));
    if (!all_equal(host, d, 0.75f, "fused pull of the pusher")) return 1;
    /* errors come back as codes, nothing was launched */
    if (dcasgd_push(h, M, g, NULL) != DCASGD_EINVAL || dcasgd_last_error(h) != DCASGD_EINVAL) return 1;
    if (dcasgd_push(h, 0, (const char*)g + 4, NULL) != DCASGD_EALIGN) return 1;
    DC_OK(dcasgd_destroy(h));

    /* 4. Supplement's fold, lambda = 1/4, eta_hat = 3/2 over J = 3 gradients (step 1/2), w_t = 0,
     *    gradients 2, 1, 4 in the caller's order:
     *      caller's order: 0 -> -1 -> -1 - (1 + 1/4*(-1))/2 = -11/8 -> -11/8 - (4 + 4*(-11/8))/2 = -5/8
     *      by ascending norm (1, 2, 4): 0 -> -1/2 -> -1/2 - (2 + 1*(-1/2))/2 = -5/4
     *                                     -> -5/4 - (4 + 4*(-5/4))/2 = -3/4 */
    {
        const float values[3] = {2.0f, 1.0f, 4.0f};
        float* grads[3] = {NULL, NULL, NULL};
        const void* list[3];
        void* workspace = NULL;
        int variant;
        for (k = 0; k < 3; ++k) {
            HIP_OK(hipMalloc((void**)&grads[k], d * sizeof(float)));
            for (i = 0; i < d; ++i) host[i] = values[k];
            HIP_OK(hipMemcpy(grads[k], host, d * sizeof(float), hipMemcpyHostToDevice));
            list[k] = grads[k];
        }
        HIP_OK(hipMalloc(&workspace, DCASGD_FOLD_WS_BYTES));
        for (variant = 0; variant < 3; ++variant) {
            memset(host, 0, d * sizeof(float));
            HIP_OK(hipMemcpy(w, host, d * sizeof(float), hipMemcpyHostToDevice));
            h = dcasgd_create(d, M, 0.5f, 0.25f, DCASGD_MODE_C, 0.0f, 0.0f);
            if (!h) { fprintf(stderr, "abi_client: dcasgd_create failed\n"); return 2; }
            DC_OK(dcasgd_bind(h, w, bak, stride, NULL));
            DC_OK(dcasgd_init(h, NULL));
            if (variant == 0) DC_OK(dcasgd_sync_fold(h, list, 3, 1.5f, NULL));
            if (variant == 1) DC_OK(dcasgd_sync_fold_ordered(h, list, 3, 1.5f, workspace, NULL));
            if (variant == 2) DC_OK(dcasgd_sync_fold_ordered_static(h, list, 3, 1.5f, NULL));
            HIP_OK(hipDeviceSynchronize());
            HIP_OK(hipMemcpy(host, w, d * sizeof(float), hipMemcpyDeviceToHost));
            if (dcasgd_step(h) != 3 ||
                !all_equal(host, d, variant == 0 ? -0.625f : -0.75f,
                           variant == 0 ? "fold in the caller's order"
                                        : variant == 1 ? "fold ranked by norm, caller's workspace"
                                                       : "fold ranked by norm, static workspace"))
                return 1;
            if (variant == 2 && dcasgd_sync_fold_ordered_static(h, list, DCASGD_MAX_K + 1, 1.5f, NULL) !=
                                    DCASGD_EINVAL)
                return 1;
            DC_OK(dcasgd_destroy(h));
        }
        HIP_OK(hipFree(workspace));
        for (k = 0; k < 3; ++k) HIP_OK(hipFree(grads[k]));
    }

    HIP_OK(hipFree(g));
    HIP_OK(hipFree(bak));
    HIP_OK(hipFree(w));
    free(host);
    printf("abi_client: OK\n");
    return 0;
}
