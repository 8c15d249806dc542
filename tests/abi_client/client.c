/* A caller of the C ABI written in plain C: no C++, no Python, no PyTorch.  Device memory comes
 * from the HIP runtime's C API.  Compresses a bf16 tensor with a ragged tail, decompresses it,
 * sums two payloads, and checks the results against what the method guarantees (Section 4.3.3:
 * the block maximum maps to the largest FP8 value, every other code is in range; the round trip
 * loses a few percent, the E4M3 rounding error; a sum of two equal payloads is twice one).
 * Exit status 0 and a line "abi_client: ok ..." on success. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "taco.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { \
    fprintf(stderr, "abi_client: %s failed: %s\n", #x, hipGetErrorString(e_)); return 2; } } while (0)
#define CHECK_TACO(x) do { int s_ = (x); if (s_ != TACO_OK) { \
    fprintf(stderr, "abi_client: %s failed: %s\n", #x, taco_strerror(s_)); return 3; } } while (0)
#define EXPECT(c) do { if (!(c)) { fprintf(stderr, "abi_client: check failed: %s (line %d)\n", #c, __LINE__); return 4; } } while (0)

static uint16_t to_bf16(float f) {
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);           /* round to nearest even */
    return (uint16_t)(u >> 16);
}

static float from_bf16(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}

static double rel_l2(const uint16_t* got, const uint16_t* ref, int64_t n, double ref_scale) {
    double num = 0.0, den = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        const double r = ref_scale * from_bf16(ref[i]), d = from_bf16(got[i]) - r;
        num += d * d;
        den += r * r;
    }
    return sqrt(num / den);
}

static int run(int32_t block, int32_t layout) {
    const int64_t rows = 37, cols = 1003, n = rows * cols;       /* 18 whole tiles of 2048 and a ragged tail */
    taco_params p;
    taco_default_params(&p);
    p.block = block;
    p.layout = layout;
    const size_t code_bytes = taco_payload_bytes(n, block), scale_bytes = taco_scales_bytes(n, block);
    EXPECT(code_bytes == (size_t)((n + block - 1) / block) * (size_t)block && scale_bytes == code_bytes / (size_t)block * 8);

    uint16_t* hx = (uint16_t*)malloc((size_t)n * 2);
    uint16_t* hout = (uint16_t*)malloc((size_t)n * 2);
    uint8_t* hpay = (uint8_t*)malloc(code_bytes + scale_bytes);
    float* hsc = (float*)malloc(scale_bytes);
    EXPECT(hx && hout && hpay && hsc);
    uint32_t state = 12345u + (uint32_t)block;
    for (int64_t i = 0; i < n; ++i) {                            /* sum of four uniforms: bell-shaped, seeded */
        float acc = 0.0f;
        for (int j = 0; j < 4; ++j) {
            state = state * 1664525u + 1013904223u;
            acc += (float)(state >> 8) * (1.0f / 16777216.0f) - 0.5f;
        }
        hx[i] = to_bf16(acc * 0.05f * ((i % 997) == 0 ? 30.0f : 1.0f));
    }

    void *dx, *dpay, *dsc, *dout;
    CHECK_HIP(hipMalloc(&dx, (size_t)n * 2));
    CHECK_HIP(hipMalloc(&dpay, code_bytes + scale_bytes));
    CHECK_HIP(hipMalloc(&dsc, scale_bytes));
    CHECK_HIP(hipMalloc(&dout, (size_t)n * 2));
    CHECK_HIP(hipMemcpy(dx, hx, (size_t)n * 2, hipMemcpyHostToDevice));

    /* argument errors come back as status codes, before any launch */
    EXPECT(taco_compress(NULL, rows, cols, &p, dpay, dsc, NULL) == TACO_ERR_NULL);
    EXPECT(taco_compress(dx, 0, cols, &p, dpay, dsc, NULL) == TACO_ERR_SHAPE);
    EXPECT(taco_compress((char*)dx + 2, rows, cols, &p, dpay, dsc, NULL) == TACO_ERR_ALIGN);
    {
        taco_params bad = p;
        bad.block = 100;
        EXPECT(taco_compress(dx, rows, cols, &bad, dpay, dsc, NULL) == TACO_ERR_BLOCK);
    }

    CHECK_TACO(taco_compress(dx, rows, cols, &p, dpay, dsc, NULL));
    CHECK_TACO(taco_decompress(dpay, dsc, rows, cols, &p, dout, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    CHECK_HIP(hipMemcpy(hout, dout, (size_t)n * 2, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(hpay, dpay, code_bytes + (layout == TACO_LAYOUT_INTERLEAVED ? scale_bytes : 0), hipMemcpyDeviceToHost));
    if (layout == TACO_LAYOUT_SPLIT) CHECK_HIP(hipMemcpy(hsc, dsc, scale_bytes, hipMemcpyDeviceToHost));

    const int64_t n_blocks = (int64_t)(code_bytes / (size_t)block);
    const int64_t rec = layout == TACO_LAYOUT_INTERLEAVED ? block + 8 : block;
    for (int64_t b = 0; b < n_blocks; ++b) {
        const uint8_t* codes = hpay + b * rec;
        float alpha, s;
        if (layout == TACO_LAYOUT_INTERLEAVED) {
            memcpy(&alpha, codes + block, 4);
            memcpy(&s, codes + block + 4, 4);
        } else {
            alpha = hsc[2 * b];
            s = hsc[2 * b + 1];
        }
        EXPECT(isfinite(alpha) && alpha > 0.0f && isfinite(s) && s >= 0.0f);
        int top = 0;
        for (int j = 0; j < block; ++j) {
            const int mag = codes[j] & 0x7F;
            EXPECT(mag != 0x7F);                                 /* never the NaN code */
            if (mag > top) top = mag;
        }
        EXPECT(s == 0.0f ? top == 0 : top == 0x7E);              /* the block maximum maps to Q_max = 448 */
    }
    const double err1 = rel_l2(hout, hx, n, 1.0);
    EXPECT(err1 > 1e-4 && err1 < 0.05);                          /* lossy, by about the E4M3 rounding error */

    const void* pays[2] = {dpay, dpay};
    const void* scs[2] = {dsc, dsc};
    CHECK_TACO(taco_decompress_sum(pays, scs, 2, rows, cols, &p, dout, NULL));
    CHECK_HIP(hipDeviceSynchronize());
    uint16_t* hsum = (uint16_t*)malloc((size_t)n * 2);
    EXPECT(hsum);
    CHECK_HIP(hipMemcpy(hsum, dout, (size_t)n * 2, hipMemcpyDeviceToHost));
    for (int64_t i = 0; i < n; ++i)                              /* x + x in fp32 then one rounding = 2 x exactly */
        EXPECT(from_bf16(hsum[i]) == 2.0f * from_bf16(hout[i]));

    CHECK_HIP(hipFree(dx));
    CHECK_HIP(hipFree(dpay));
    CHECK_HIP(hipFree(dsc));
    CHECK_HIP(hipFree(dout));
    free(hx); free(hout); free(hpay); free(hsc); free(hsum);
    printf("abi_client: block %d layout %d: %lld blocks, round-trip relative L2 error %.4f\n", block, layout,
           (long long)n_blocks, err1);
    return 0;
}

int main(void) {
    printf("abi_client: library version %s\n", taco_version());
    const int32_t blocks[5] = {32, 64, 128, 256, 512};
    for (int i = 0; i < 5; ++i)
        for (int32_t layout = 0; layout < 2; ++layout) {
            const int rc = run(blocks[i], layout);
            if (rc != 0) return rc;
        }
    printf("abi_client: ok\n");
    return 0;
}
