/*
 * A plain C program that uses libbittrain through its C ABI only (no Python, no torch):
 * device buffers from the HIP runtime, every call checked against the C oracle that is
 * linked in (test infrastructure).  Prints "c_client ok" and returns 0 on success.
 *
 * Built by __graft_entry__.build() with hipcc; run by tests/test_gpu_z_c_client.py.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "bittrain.h"

uint64_t bt_oracle_compress(const void *T, uint64_t n, int width, uint32_t *bitmap, void *values);
uint64_t bt_oracle_decompress(const uint32_t *bitmap, const void *values, uint64_t n, int width, void *T);
int bt_oracle_relu_backward(const uint32_t *bitmap, const void *grad_out, uint64_t n, int width, void *grad_in);
uint64_t bt_oracle_compressed_size(uint64_t n, uint64_t nnz, int width);

#define HIP_OK(call)                                                                        \
    do {                                                                                    \
        hipError_t e_ = (call);                                                             \
        if (e_ != hipSuccess) {                                                             \
            fprintf(stderr, "%s failed: %s (line %d)\n", #call, hipGetErrorString(e_), __LINE__); \
            return 2;                                                                       \
        }                                                                                   \
    } while (0)
#define BT_OK_OR_FAIL(call)                                                                 \
    do {                                                                                    \
        bt_status s_ = (call);                                                              \
        if (s_ != BT_OK) {                                                                  \
            fprintf(stderr, "%s failed: %s (line %d)\n", #call, bt_status_str(s_), __LINE__); \
            return 3;                                                                       \
        }                                                                                   \
    } while (0)

/* xorshift: the inputs only have to be reproducible */
static uint32_t rng_state = 2463534242u;
static uint32_t rng(void)
{
    rng_state ^= rng_state << 13;
    rng_state ^= rng_state >> 17;
    rng_state ^= rng_state << 5;
    return rng_state;
}

static int run(uint64_t n, bt_dtype dtype, int width, unsigned zero_per_256)
{
    const size_t bytes = (size_t)n * (size_t)width, words = (size_t)((n + 31) / 32);
    unsigned char *x = (unsigned char *)malloc(bytes + 8), *g = (unsigned char *)malloc(bytes + 8);
    unsigned char *got = (unsigned char *)malloc(bytes + 8), *want = (unsigned char *)malloc(bytes + 8);
    uint32_t *o_bitmap = (uint32_t *)malloc(4 * words + 4), *h_bitmap = (uint32_t *)malloc(4 * words + 4);
    unsigned char *o_values = (unsigned char *)malloc(bytes + 8), *h_values = (unsigned char *)malloc(bytes + 8);
    if (!x || !g || !got || !want || !o_bitmap || !h_bitmap || !o_values || !h_values) return 4;
    for (uint64_t i = 0; i < n; ++i) {
        uint64_t v = ((uint64_t)rng() << 32) | rng();
        if ((rng() & 255u) < zero_per_256) v = 0;
        memcpy(x + i * (size_t)width, &v, (size_t)width);
        uint64_t w = ((uint64_t)rng() << 32) | rng();
        memcpy(g + i * (size_t)width, &w, (size_t)width);
    }
    const uint64_t o_nnz = bt_oracle_compress(x, n, width, o_bitmap, o_values);

    void *d_x, *d_values, *d_out, *d_g, *d_ws;
    uint32_t *d_bitmap;
    uint64_t *d_nnz, h_nnz = ~(uint64_t)0;
    const size_t ws_bytes = bt_workspace_bytes(n, dtype);
    HIP_OK(hipMalloc(&d_x, bytes + 16));
    HIP_OK(hipMalloc(&d_values, bytes + 16));
    HIP_OK(hipMalloc(&d_out, bytes + 16));
    HIP_OK(hipMalloc(&d_g, bytes + 16));
    HIP_OK(hipMalloc((void **)&d_bitmap, 4 * words + 16));
    HIP_OK(hipMalloc((void **)&d_nnz, 8));
    HIP_OK(hipMalloc(&d_ws, ws_bytes));
    HIP_OK(hipMemcpy(d_x, x, bytes, hipMemcpyHostToDevice));
    HIP_OK(hipMemcpy(d_g, g, bytes, hipMemcpyHostToDevice));
    hipStream_t stream;
    HIP_OK(hipStreamCreate(&stream));

    BT_OK_OR_FAIL(bt_workspace_init(d_ws, ws_bytes, stream));
    BT_OK_OR_FAIL(bt_compress(d_x, n, dtype, d_bitmap, d_values, n, d_nnz, d_ws, ws_bytes, stream));
    BT_OK_OR_FAIL(bt_decompress(d_bitmap, d_values, n, dtype, d_out, d_ws, ws_bytes, stream));
    BT_OK_OR_FAIL(bt_relu_backward_from_bitmap(d_bitmap, d_g, n, dtype, d_g, stream));   /* in place */
    HIP_OK(hipStreamSynchronize(stream));

    HIP_OK(hipMemcpy(&h_nnz, d_nnz, 8, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(h_bitmap, d_bitmap, 4 * words, hipMemcpyDeviceToHost));
    HIP_OK(hipMemcpy(h_values, d_values, bytes, hipMemcpyDeviceToHost));
    int bad = 0;
    if (h_nnz != o_nnz) { fprintf(stderr, "nnz %llu != %llu\n", (unsigned long long)h_nnz, (unsigned long long)o_nnz); bad = 1; }
    if (memcmp(h_bitmap, o_bitmap, 4 * words) != 0) { fprintf(stderr, "bitmap differs\n"); bad = 1; }
    if (memcmp(h_values, o_values, (size_t)o_nnz * (size_t)width) != 0) { fprintf(stderr, "values differ\n"); bad = 1; }
    if (bt_compressed_size(n, h_nnz, dtype) != bt_oracle_compressed_size(n, o_nnz, width)) { fprintf(stderr, "size differs\n"); bad = 1; }
    HIP_OK(hipMemcpy(got, d_out, bytes, hipMemcpyDeviceToHost));
    bt_oracle_decompress(o_bitmap, o_values, n, width, want);
    if (memcmp(got, want, bytes) != 0 || memcmp(got, x, bytes) != 0) { fprintf(stderr, "restored tensor differs\n"); bad = 1; }
    HIP_OK(hipMemcpy(got, d_g, bytes, hipMemcpyDeviceToHost));
    bt_oracle_relu_backward(o_bitmap, g, n, width, want);
    if (memcmp(got, want, bytes) != 0) { fprintf(stderr, "relu backward differs\n"); bad = 1; }

    HIP_OK(hipStreamDestroy(stream));
    HIP_OK(hipFree(d_x)); HIP_OK(hipFree(d_values)); HIP_OK(hipFree(d_out)); HIP_OK(hipFree(d_g));
    HIP_OK(hipFree(d_bitmap)); HIP_OK(hipFree(d_nnz)); HIP_OK(hipFree(d_ws));
    free(x); free(g); free(got); free(want); free(o_bitmap); free(h_bitmap); free(o_values); free(h_values);
    printf("n=%llu width=%d nnz=%llu %s\n", (unsigned long long)n, width, (unsigned long long)o_nnz, bad ? "MISMATCH" : "ok");
    return bad;
}

int main(void)
{
    int bad = 0;
    bad |= run(1, BT_F32, 4, 0);
    bad |= run(200704, BT_F32, 4, 128);
    bad |= run(3 * 16384 + 77, BT_BF16, 2, 200);
    bad |= run(70 * 8192 + 5, BT_F32, 4, 64);
    bad |= run(33 * 4096 + 1, BT_F64, 8, 128);
    bad |= run(1000003, BT_F16, 2, 250);
    if (bad) return 1;
    printf("c_client ok\n");
    return 0;
}
