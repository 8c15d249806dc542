// Plain butterfly kernels: one 64-lane wavefront per block of B elements, any supported B
// (32 .. 512), any n (ragged tails are bounds-checked).  They serve block sizes without a
// matrix-core kernel and the tail of a tensor that does not fill a whole tile.
//
// Element e of a block lives in lane (e & 63), register (e >> 6).  The fast Walsh-Hadamard
// transform (Algorithm 1, sender and receiver sides) then splits into stages that
// exchange values between lanes (strides 1 .. 32, a wave shuffle) and stages between
// registers of one lane (strides 64 and up).  The in-place butterfly with stride h maps
// (a, b) -> (a + b, a - b) for the pair whose indices differ in bit h; running all strides
// gives y = H x with H[i][j] = (-1)^popcount(i & j), the natural ordering.
//
// The transform runs on the raw block (bf16 inputs, or decoded FP8 codes) so that most
// partial sums are exact in fp32, and the block scalars are applied once afterwards
// (the rotation is linear, so alpha_k and 1/sqrt(B) commute with it).
#pragma once

#include "device_util.h"

namespace taco {

template <int B>
struct ButterflyShape {
    static constexpr int kRegs = (B + 63) / 64;   // values per lane
    static constexpr int kLanes = B < 64 ? B : 64;  // lanes that hold data
};

// y = H x over the wave; v[r] holds element lane + 64 r.  Lanes >= B (B = 32) carry zeros.
template <int B>
__device__ __forceinline__ void fwht_wave(float (&v)[ButterflyShape<B>::kRegs], int lane) {
    constexpr int R = ButterflyShape<B>::kRegs;
#pragma unroll
    for (int h = 1; h < 64 && h < B; h <<= 1) {
        const bool upper = (lane & h) != 0;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float other = __shfl_xor(v[r], h, 64);
            v[r] = upper ? other - v[r] : v[r] + other;
        }
    }
#pragma unroll
    for (int hr = 1; hr < R; hr <<= 1) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            if ((r & hr) == 0) {
                float a = v[r], b = v[r | hr];
                v[r] = a + b;
                v[r | hr] = a - b;
            }
        }
    }
}

// Ablation variants (the paper's component and format ablations): a stage switched off or another
// code book.  mode bits: 1 adaptive rescaling, 2 Hadamard rotation, 4 post-rotation scale; formats:
// 0 E4M3, 1 E5M2, 2 INT8 (round(x / Delta), Delta = max|x| / 127).  7 and 0 are the method itself.
struct Variant {
    int mode;
    int format;
    __device__ __forceinline__ bool rescale() const { return (mode & 1) != 0; }
    __device__ __forceinline__ bool rotate() const { return (mode & 2) != 0; }
    __device__ __forceinline__ bool postscale() const { return (mode & 4) != 0; }
    __device__ __forceinline__ float qmax() const { return format == 0 ? 448.0f : format == 1 ? 57344.0f : 127.0f; }
};

__device__ __forceinline__ uint8_t encode_value(float q, const Variant& var) {
    if (var.format == 0) return static_cast<uint8_t>(__builtin_amdgcn_cvt_pk_fp8_f32(q, q, 0, false) & 0xFF);
    if (var.format == 1) return static_cast<uint8_t>(__builtin_amdgcn_cvt_pk_bf8_f32(q, q, 0, false) & 0xFF);
    return static_cast<uint8_t>(static_cast<int8_t>(static_cast<int>(__builtin_rintf(q))));
}

__device__ __forceinline__ float decode_value(uint8_t code, const Variant& var) {
    if (var.format == 0) return __builtin_amdgcn_cvt_f32_fp8(code, 0);
    if (var.format == 1) return __builtin_amdgcn_cvt_f32_bf8(code, 0);
    return static_cast<float>(static_cast<int8_t>(code));
}

// Byte offset of block blk's codes in the payload buffer: blocks are B bytes apart in the split
// layout and B + 8 bytes apart (codes, then {alpha, s}) in the interleaved one.
template <int B>
__device__ __forceinline__ int64_t code_offset(int64_t blk, bool interleaved) {
    return blk * (interleaved ? B + 8 : B);
}

// Sender side of Algorithm 1 for one block whose elements are already in registers
// (v[r] = element lane + 64 r, zeros past the end of the tensor).
template <int B>
__device__ __forceinline__ void compress_block_butterfly(float (&v)[ButterflyShape<B>::kRegs], int lane, int64_t blk,
                                                         float tau, float eps, uint8_t* __restrict__ payload,
                                                         float2* __restrict__ scales, bool interleaved, Variant var) {
    constexpr int R = ButterflyShape<B>::kRegs;
    float alpha = 1.0f;
    if (var.rescale()) {
        float energy = 0.0f;
#pragma unroll
        for (int r = 0; r < R; ++r) energy = __builtin_fmaf(v[r], v[r], energy);
        energy = wave_allreduce_sum(energy);                          // sum_j G_kj^2
        alpha = tau * __builtin_amdgcn_rsqf(energy * (1.0f / B) + eps);   // Eq. ash_sigma, Eq. ash_alpha
    }
    float norm = 1.0f;
    if (var.rotate()) {
        fwht_wave<B>(v, lane);                                        // W = H G_k (unnormalised)
        norm = 1.0f / __builtin_sqrtf(static_cast<float>(B));
    }
    float wmax = 0.0f;
#pragma unroll
    for (int r = 0; r < R; ++r) wmax = fmaxf(wmax, __builtin_fabsf(v[r]));
    wmax = wave_allreduce_max(wmax);
    const float qmax = var.qmax();
    // Z = alpha W / sqrt(B); with the post-rotation scale, s = max|Z| / Q_max (Eq. post_scale) and
    // Z / s = Q_max W / max|W| in exact arithmetic (zero blocks map to zero codes); without it s = 1
    // and Z itself is converted, saturating at +-Q_max.
    float s = 1.0f, to_code = alpha * norm;
    if (var.postscale()) {
        s = wmax > 0.0f ? (wmax * alpha * norm) * (1.0f / qmax) : 0.0f;   // all-zero block: s = 0 even if alpha is infinite (eps = 0)
        to_code = wmax > 0.0f ? qmax * __builtin_amdgcn_rcpf(wmax) : 0.0f;
    }
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const int e = lane + 64 * r;
        if (e < B) {
            float q = v[r] * to_code;
            if (!var.postscale() || var.format == 2) q = __builtin_amdgcn_fmed3f(q, -qmax, qmax);
            payload[code_offset<B>(blk, interleaved) + e] = encode_value(q, var);
        }
    }
    if (lane == 0) {
        if (interleaved) *reinterpret_cast<float2*>(payload + code_offset<B>(blk, true) + B) = make_float2(alpha, s);
        else scales[blk] = make_float2(alpha, s);
    }
}

// Sender side of Algorithm 1 for blocks [first_block, first_block + n_blocks).
template <int B>
__global__ __launch_bounds__(64) void compress_butterfly_kernel(
    const uint16_t* __restrict__ x, int64_t n, int64_t first_block, int64_t n_blocks, float tau,
    float eps, uint8_t* __restrict__ payload, float2* __restrict__ scales, bool interleaved, Variant var) {
    constexpr int R = ButterflyShape<B>::kRegs;
    const int lane = threadIdx.x;
    for (int64_t blk = first_block + blockIdx.x; blk < first_block + n_blocks; blk += gridDim.x) {
        float v[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int e = lane + 64 * r;
            const int64_t idx = blk * B + e;
            v[r] = (e < B && idx < n) ? bf16_bits_to_f32(x[idx]) : 0.0f;   // zero padding
        }
        compress_block_butterfly<B>(v, lane, blk, tau, eps, payload, scales, interleaved, var);
    }
}

struct PayloadTable {
    const void* payload[16];
    const void* scales[16];
};

// Receiver side of Algorithm 1 plus the local reduction over k payloads for one block; the
// result (before the final rounding to bf16) is left in v.  The rotation is linear, so for
// k > 1 the codes are first combined with their block factors s / (alpha sqrt(B)) and rotated
// once; for k = 1 the raw codes are rotated (exact partial sums) and the factor is applied
// afterwards.
template <int B>
__device__ __forceinline__ void decode_sum_block_butterfly(const PayloadTable& tab, int k, int64_t blk, int lane,
                                                           float (&v)[ButterflyShape<B>::kRegs], bool interleaved,
                                                           Variant var) {
    constexpr int R = ButterflyShape<B>::kRegs;
    const float inv_root_b = var.rotate() ? 1.0f / __builtin_sqrtf(static_cast<float>(B)) : 1.0f;
#pragma unroll
    for (int r = 0; r < R; ++r) v[r] = 0.0f;
    float single = 1.0f;
    for (int i = 0; i < k; ++i) {
        const uint8_t* codes = static_cast<const uint8_t*>(tab.payload[i]) + code_offset<B>(blk, interleaved);
        const float2 sc = interleaved ? *reinterpret_cast<const float2*>(codes + B)
                                      : static_cast<const float2*>(tab.scales[i])[blk];
        const float factor = sc.y * __builtin_amdgcn_rcpf(sc.x) * inv_root_b;   // s / (alpha sqrt(B))
        const float w = (k == 1) ? 1.0f : factor;
        single = factor;
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int e = lane + 64 * r;
            if (e < B) {
                const float q = decode_value(codes[e], var);
                v[r] = __builtin_fmaf(q, w, v[r]);
            }
        }
    }
    if (var.rotate()) fwht_wave<B>(v, lane);
    const float post = (k == 1) ? single : 1.0f;
#pragma unroll
    for (int r = 0; r < R; ++r) v[r] *= post;
}

template <int B>
__global__ __launch_bounds__(64) void decompress_sum_butterfly_kernel(
    PayloadTable tab, int k, int64_t n, int64_t first_block, int64_t n_blocks,
    uint16_t* __restrict__ out, bool interleaved, Variant var) {
    constexpr int R = ButterflyShape<B>::kRegs;
    const int lane = threadIdx.x;
    for (int64_t blk = first_block + blockIdx.x; blk < first_block + n_blocks; blk += gridDim.x) {
        float v[R];
        decode_sum_block_butterfly<B>(tab, k, blk, lane, v, interleaved, var);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int e = lane + 64 * r;
            const int64_t idx = blk * B + e;
            if (e < B && idx < n) out[idx] = static_cast<uint16_t>(pack_bf16x2(v[r], 0.0f) & 0xFFFF);
        }
    }
}

// decompress_sum followed by compress of the bf16-rounded sum, block by block, without the
// bf16 tensor leaving the registers.
template <int B>
__global__ __launch_bounds__(64) void decompress_sum_compress_butterfly_kernel(
    PayloadTable tab, int k, int64_t n, int64_t first_block, int64_t n_blocks, float tau, float eps,
    uint8_t* __restrict__ payload_out, float2* __restrict__ scales_out, bool interleaved, Variant var) {
    constexpr int R = ButterflyShape<B>::kRegs;
    const int lane = threadIdx.x;
    for (int64_t blk = first_block + blockIdx.x; blk < first_block + n_blocks; blk += gridDim.x) {
        float v[R];
        decode_sum_block_butterfly<B>(tab, k, blk, lane, v, interleaved, var);
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int e = lane + 64 * r;
            const int64_t idx = blk * B + e;
            v[r] = (e < B && idx < n) ? bf16_bits_to_f32(pack_bf16x2(v[r], 0.0f) & 0xFFFF) : 0.0f;
        }
        compress_block_butterfly<B>(v, lane, blk, tau, eps, payload_out, scales_out, interleaved, var);
    }
}

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
__global__ __launch_bounds__(64 * kWaves) void traffic_kernel(PayloadTable srcs, int k, int src_chunks,
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
                const u32x4* src = static_cast<const u32x4*>(srcs.payload[i0 + j]) + tile * src_chunks;
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
