// Diagnostic kernels behind include/taco_debug.h: the hardware FP8 conversion on its own, a plain
// copy, and the operator's memory traffic without its arithmetic.  Not part of the operator.
#pragma once

#include "device_util.h"
#include "tables.h"

namespace taco {

struct SourceTable {
    const void* src[kMaxK];
};

// Hardware float -> E4M3 conversion, one value per thread (diagnostic entry point).
__global__ void cvt_e4m3_kernel(const float* __restrict__ in, int64_t n, uint8_t* __restrict__ out) {
    int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x;
    if (i < n) {
        const float v = in[i];
        out[i] = static_cast<uint8_t>(__builtin_amdgcn_cvt_pk_fp8_f32(v, v, 0, false) & 0xFF);
    }
}

// Plain copy, 16 bytes per lane, grid-stride (diagnostic entry point).
__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t n16) {
    const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}

// The operator's memory traffic without its arithmetic (diagnostic entry point): wave v reads
// src_chunks 16-byte words of tile v from each of k sources and writes dst_chunks words of tile v,
// with the non-temporal loads and stores and the one-shot launch shape of the matrix-core kernels.
// The written words are XORs of the loaded ones, so no load can be dropped.
template <int kWaves>
__global__ __launch_bounds__(64 * kWaves) void traffic_kernel(SourceTable srcs, int k, int src_chunks,
                                                              u32x4* __restrict__ dst, int dst_chunks, int64_t n_tiles) {
    const int lane = threadIdx.x & 63;
    const int64_t tile = static_cast<int64_t>(blockIdx.x) * kWaves + (threadIdx.x >> 6);
    if (tile >= n_tiles) return;
    u32x4 acc[4] = {u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}, u32x4{0, 0, 0, 0}};
    for (int i0 = 0; i0 < k; i0 += 4) {
        u32x4 v[4][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int c = 0; c < 4; ++c) v[j][c] = u32x4{0, 0, 0, 0};
            if (i0 + j < k) {
                const u32x4* src = static_cast<const u32x4*>(srcs.src[i0 + j]) + tile * src_chunks;
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    if (64 * c + lane < src_chunks) v[j][c] = load16<true>(&src[64 * c + lane]);
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
            for (int c = 0; c < 4; ++c) acc[c] ^= v[j][c];
        }
    }
    acc[0] ^= acc[2];
    acc[1] ^= acc[3];
    acc[2] ^= acc[1];
    acc[3] ^= acc[0];
    u32x4* out = dst + tile * dst_chunks;
#pragma unroll
    for (int c = 0; c < 4; ++c)
        if (64 * c + lane < dst_chunks) store_stream<true>(&out[64 * c + lane], acc[c]);
}

}  // namespace taco
