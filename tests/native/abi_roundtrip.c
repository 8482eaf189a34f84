/*
 * The C ABI of include/l3.h used from plain C, with nothing but the HIP runtime beside
 * it: encode an image on the host, copy the file to the GPU, decode it there, compare.
 * Built by paper_2208_08711_amd/build.py next to libl3.so; run by a GPU test.
 * Exit status 0 = the decoded pixels equal the input.
 */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <hip/hip_runtime_api.h>

#include "l3.h"

#define CHECK_HIP(call)                                                        \
    do {                                                                       \
        hipError_t e_ = (call);                                                \
        if (e_ != hipSuccess) {                                                \
            fprintf(stderr, "%s: %s\n", #call, hipGetErrorString(e_));         \
            return 2;                                                          \
        }                                                                      \
    } while (0)

#define CHECK_L3(call)                                                         \
    do {                                                                       \
        l3_status s_ = (call);                                                 \
        if (s_ != L3_OK) {                                                     \
            fprintf(stderr, "%s: %s\n", #call, l3_status_string(s_));          \
            return 3;                                                          \
        }                                                                      \
    } while (0)

int main(void) {
    const uint32_t w = 301, h = 157;
    uint8_t* rgb = (uint8_t*)malloc((size_t)w * h * 3);
    uint32_t state = 12345u;
    for (uint32_t y = 0; y < h; ++y)
        for (uint32_t x = 0; x < w; ++x)
            for (uint32_t c = 0; c < 3; ++c) {
                state = state * 1664525u + 1013904223u;
                rgb[((size_t)y * w + x) * 3 + c] = (uint8_t)(40 + x / 2 + y / 3 + 20 * c + ((state >> 24) & 7));
            }

    const size_t cap = l3_encode_bound(w, h, 0);
    uint8_t* file = (uint8_t*)malloc(cap);
    size_t len = 0;
    CHECK_L3(l3_encode_cpu(rgb, w, h, (size_t)w * 3, 0, file, cap, &len));
    l3_info info;
    CHECK_L3(l3_peek_header(file, len, &info));
    if (info.width != w || info.height != h || info.patch != l3_default_patch(w, h)) return 4;

    uint8_t *d_file = NULL, *d_out = NULL;
    uint32_t* d_status = NULL;
    CHECK_HIP(hipMalloc((void**)&d_file, len));
    CHECK_HIP(hipMalloc((void**)&d_out, (size_t)w * h * 3));
    CHECK_HIP(hipMalloc((void**)&d_status, sizeof(uint32_t)));
    CHECK_HIP(hipMemcpy(d_file, file, len, hipMemcpyHostToDevice));

    l3_ctx* ctx = NULL;
    CHECK_L3(l3_ctx_create(&ctx, 0));
    l3_item item;
    memset(&item, 0, sizeof item);
    item.d_file = d_file;
    item.file_len = len;
    item.info = info;
    item.d_out = d_out;
    item.out_row_stride = (size_t)w * 3;
    CHECK_L3(l3_decode_batch(ctx, &item, 1, L3_LAYOUT_HWC, d_status, NULL));
    CHECK_HIP(hipDeviceSynchronize());

    uint8_t* back = (uint8_t*)malloc((size_t)w * h * 3);
    uint32_t status = 99;
    CHECK_HIP(hipMemcpy(back, d_out, (size_t)w * h * 3, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(&status, d_status, sizeof status, hipMemcpyDeviceToHost));
    l3_ctx_destroy(ctx);
    CHECK_HIP(hipFree(d_file));
    CHECK_HIP(hipFree(d_out));
    CHECK_HIP(hipFree(d_status));

    if (status != 0) {
        fprintf(stderr, "status word %u\n", status);
        return 5;
    }
    if (memcmp(back, rgb, (size_t)w * h * 3) != 0) {
        fprintf(stderr, "decoded pixels differ\n");
        return 6;
    }
    printf("abi_roundtrip ok: %u x %u, %zu file bytes (%.3f of raw)\n", w, h, len,
           (double)len / ((double)w * h * 3));
    free(rgb);
    free(file);
    free(back);
    return 0;
}
