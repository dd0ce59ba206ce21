/* A plain C99 caller of libfcdp that does GPU work: it allocates device and
 * pinned host memory through the HIP runtime's C API, calls the data entry
 * points with plain pointers, and checks the bytes against values it works
 * out itself from the definition (tensor_t[j] = flat[off_t + j]; the reduced
 * element = p_0 + p_1 + p_2 in that order).  Built and run by
 * tests/test_c_abi.py on a machine with a GPU. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "fcdp.h"

#define CHECK(cond)                                                           \
    do {                                                                      \
        if (!(cond)) {                                                        \
            printf("FAILED line %d: %s (last error: %s)\n", __LINE__, #cond,  \
                   fcdp_last_error());                                        \
            return 1;                                                         \
        }                                                                     \
    } while (0)

int main(void)
{
    enum { T = 3, G = 4 };
    const int64_t numel[T] = {5000, 37, 12001};
    fcdp_layout *L = NULL;
    int64_t N, Np, S, t, j, r;
    uint16_t *flat, *back;
    void *d_shards[G], *d_tensors[T], *d_staging, *host = NULL, *alias = NULL;
    const void *shard_ptrs[G];
    void *tensor_ptrs[T];
    hipStream_t compute, copy;
    const int64_t *off;

    CHECK(fcdp_layout_build(numel, NULL, T, G, 2, 64, &L) == FCDP_OK);
    CHECK(fcdp_layout_prepare(L) == FCDP_OK);
    N = fcdp_layout_numel(L);
    Np = fcdp_layout_padded_numel(L);
    S = fcdp_layout_shard_numel(L);
    off = fcdp_layout_offsets(L);
    CHECK(N == 17038 && Np % (G * 64) == 0 && S * G == Np);
    flat = (uint16_t *)calloc((size_t)Np, 2);
    back = (uint16_t *)malloc((size_t)Np * 2);
    CHECK(flat && back);
    for (j = 0; j < N; ++j) flat[j] = (uint16_t)(j * 40503u + 7u);
    CHECK(hipStreamCreate(&compute) == hipSuccess && hipStreamCreate(&copy) == hipSuccess);
    for (r = 0; r < G; ++r) {
        CHECK(hipMalloc(&d_shards[r], (size_t)S * 2) == hipSuccess);
        CHECK(hipMemcpy(d_shards[r], flat + r * S, (size_t)S * 2, hipMemcpyHostToDevice) == hipSuccess);
        shard_ptrs[r] = d_shards[r];
    }
    for (t = 0; t < T; ++t) {
        CHECK(hipMalloc(&d_tensors[t], (size_t)numel[t] * 2 + 16) == hipSuccess);
        CHECK(hipMemset(d_tensors[t], 0xC3, (size_t)numel[t] * 2 + 16) == hipSuccess);
        tensor_ptrs[t] = d_tensors[t];
    }
    CHECK(hipMalloc(&d_staging, (size_t)Np * 2) == hipSuccess);
    CHECK(fcdp_host_cache_alloc((size_t)Np * 2, -1, &host, &alias) == FCDP_OK);
    memset(host, 0xEE, (size_t)Np * 2);

    /* forward: scatter the shards, store the image to the host cache */
    CHECK(fcdp_materialize_layer(L, FCDP_SRC_DEVICE_SHARDS, shard_ptrs, host, NULL, tensor_ptrs,
                                 FCDP_STORE_DMA, compute, copy) == FCDP_OK);
    CHECK(hipDeviceSynchronize() == hipSuccess);
    CHECK(memcmp(host, flat, (size_t)Np * 2) == 0);
    for (t = 0; t < T; ++t) {
        CHECK(hipMemcpy(back, d_tensors[t], (size_t)numel[t] * 2 + 16, hipMemcpyDeviceToHost) == hipSuccess);
        CHECK(memcmp(back, flat + off[t], (size_t)numel[t] * 2) == 0);
        for (j = 0; j < 16; ++j) CHECK(((unsigned char *)back)[numel[t] * 2 + j] == 0xC3);
        CHECK(hipMemset(d_tensors[t], 0, (size_t)numel[t] * 2) == hipSuccess);
    }
    /* backward: staged fetch, then the allocation-free variant, then zero-copy */
    for (r = 0; r < 3; ++r) {
        fcdp_status st = r == 0 ? fcdp_materialize_layer(L, FCDP_SRC_HOST_DMA, NULL, host, d_staging, tensor_ptrs,
                                                         FCDP_STORE_NONE, compute, copy)
                         : r == 1 ? fcdp_materialize_layer_static(L, host, tensor_ptrs, compute, copy)
                                  : fcdp_materialize_layer(L, FCDP_SRC_HOST_ZEROCOPY, NULL, host, NULL, tensor_ptrs,
                                                           FCDP_STORE_NONE, compute, copy);
        CHECK(st == FCDP_OK);
        CHECK(hipDeviceSynchronize() == hipSuccess);
        for (t = 0; t < T; ++t) {
            CHECK(hipMemcpy(back, d_tensors[t], (size_t)numel[t] * 2, hipMemcpyDeviceToHost) == hipSuccess);
            CHECK(memcmp(back, flat + off[t], (size_t)numel[t] * 2) == 0);
            CHECK(hipMemset(d_tensors[t], 0, (size_t)numel[t] * 2) == hipSuccess);
        }
    }
    /* pageable memory is refused, and nothing is left in an error state */
    CHECK(fcdp_materialize_layer(L, FCDP_SRC_HOST_DMA, NULL, flat, d_staging, tensor_ptrs,
                                 FCDP_STORE_NONE, compute, copy) == FCDP_ENOTPINNED);
    {
        /* gradient shard: three partials, sum in rank order */
        enum { R = 3, C = 4099 };
        float *p[R], *sum = (float *)malloc(C * sizeof(float)), *got = (float *)malloc(C * sizeof(float));
        void *d_p[R], *d_out;
        const void *pp[R];
        int k;
        CHECK(sum && got);
        for (k = 0; k < R; ++k) {
            p[k] = (float *)malloc(C * sizeof(float));
            CHECK(p[k] != NULL);
            for (j = 0; j < C; ++j) p[k][j] = (float)((j * 7 + k * 13) % 1000) * (k == 1 ? 1e-3f : 3.0f) - 100.0f;
            CHECK(hipMalloc(&d_p[k], C * sizeof(float)) == hipSuccess);
            CHECK(hipMemcpy(d_p[k], p[k], C * sizeof(float), hipMemcpyHostToDevice) == hipSuccess);
            pp[k] = d_p[k];
        }
        for (j = 0; j < C; ++j) {
            volatile float a = p[0][j];
            a = a + p[1][j];
            a = a + p[2][j];
            sum[j] = a;
        }
        CHECK(hipMalloc(&d_out, C * sizeof(float)) == hipSuccess);
        CHECK(fcdp_reduce_grad_shard(pp, R, 0, C, FCDP_F32, FCDP_F32, d_out, compute) == FCDP_OK);
        CHECK(hipDeviceSynchronize() == hipSuccess);
        CHECK(hipMemcpy(got, d_out, C * sizeof(float), hipMemcpyDeviceToHost) == hipSuccess);
        CHECK(memcmp(got, sum, C * sizeof(float)) == 0);
        for (k = 0; k < R; ++k) {
            free(p[k]);
            (void)hipFree(d_p[k]);
        }
        (void)hipFree(d_out);
        free(sum);
        free(got);
    }
    CHECK(fcdp_host_cache_free(host) == FCDP_OK);
    for (r = 0; r < G; ++r) (void)hipFree(d_shards[r]);
    for (t = 0; t < T; ++t) (void)hipFree(d_tensors[t]);
    (void)hipFree(d_staging);
    fcdp_layout_destroy(L);
    free(flat);
    free(back);
    printf("c abi gpu ok\n");
    return 0;
}
