// Plain butterfly kernels, any supported B (32 .. 512) and any n (ragged tails are bounds-checked).
// They serve the part of a tensor that does not fill a whole tile of the matrix-core kernels, the
// run-time selectable ablation variants, and impl = BUTTERFLY as a second, independent family.
//
// A wave works on a TILE of 2048 consecutive elements (the same unit of work as the matrix-core
// kernels: one single-wave workgroup per tile, no persistent loop) as four GROUPS of 512 elements =
// 512 / B whole blocks each: lane L holds the eight elements 8 L .. 8 L + 7 of a group (one 16-byte
// load of bf16, one 8-byte load or store of codes), so a block occupies B / 8 neighbouring lanes.
// The loads of all four groups are issued before the first is used; loads and stores are
// non-temporal (every byte is touched once).  The fast Walsh-Hadamard transform
// (Algorithm 1, sender and receiver sides) then splits into three stages between the registers of
// a lane (strides 1, 2, 4) and log2(B / 8) stages that exchange values between lanes L and L ^ m.
// The in-place butterfly with stride h maps (a, b) -> (a + b, a - b) for the pair whose indices
// differ in bit h; running all strides gives y = H x with H[i][j] = (-1)^popcount(i & j), the
// natural ordering.  Sums and maxima over a block are xor-shuffle reductions over the same lanes.
//
// The transform runs on the raw block (bf16 inputs, or decoded FP8 codes) so that most
// partial sums are exact in fp32, and the block scalars are applied once afterwards
// (the rotation is linear, so alpha_k and 1/sqrt(B) commute with it).
#pragma once

#include "device_util.h"
#include "tables.h"

namespace taco {

constexpr int kGroupElems = 512;      // elements whose transform one wave holds in registers at a time
constexpr int kGroupsPerTile = 4;     // groups per wave: one tile of 2048 elements

// Butterfly between lanes L and L ^ kMask (element stride 8 kMask); nothing when the block is narrower.
// The lower lane of a pair wants a + b and the upper one a - b (a the lower lane's value).  Written as
// own + sgn * other with sgn = +1 in the lower and -1 in the upper lane, the upper lane gets b - a, the result
// with its sign flipped, in ONE instruction per value (a multiply-add whose operand comes through the
// cross-lane path) instead of a move, two additions and a select.  The flipped signs need no bookkeeping
// between stages: partner lanes differ only in the bit of the current stage, so they have been flipped
// equally often before it; after all stages lane L carries (-1)^popcount(L & (B/8 - 1)) times the
// transform, which fwht_group returns for the caller to fold into the factor it multiplies by anyway.
// Products with +-1 are exact, so every value is the one the plain butterfly would give.
template <int B, int kMask>
__device__ __forceinline__ void cross_lane_stage(float (&v)[8], int lane) {
    if (kMask < B / 8) {
        const float sgn = (lane & kMask) != 0 ? -1.0f : 1.0f;
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] = __builtin_fmaf(sgn, lane_xor<kMask>(v[r]), v[r]);
    }
}

// y = H_B x for every block of the group, up to the sign that is returned: v[r] * sign is element 8 lane + r of y.
template <int B>
__device__ __forceinline__ float fwht_group(float (&v)[8], int lane) {
#pragma unroll
    for (int h = 1; h < 8; h <<= 1) {
#pragma unroll
        for (int r = 0; r < 8; ++r) {
            if ((r & h) == 0) {
                const float a = v[r], b = v[r | h];
                v[r] = a + b;
                v[r | h] = a - b;
            }
        }
    }
    cross_lane_stage<B, 1>(v, lane);
    cross_lane_stage<B, 2>(v, lane);
    cross_lane_stage<B, 4>(v, lane);
    cross_lane_stage<B, 8>(v, lane);
    cross_lane_stage<B, 16>(v, lane);
    cross_lane_stage<B, 32>(v, lane);
    return (__builtin_popcount(lane & (B / 8 - 1)) & 1) ? -1.0f : 1.0f;
}

// Sum / maximum over the B / 8 lanes of the caller's block, returned in every one of them.
template <int B>
__device__ __forceinline__ float block_allreduce_sum(float v) {
    if (1 < B / 8) v += lane_xor<1>(v);
    if (2 < B / 8) v += lane_xor<2>(v);
    if (4 < B / 8) v += lane_xor<4>(v);
    if (8 < B / 8) v += lane_xor<8>(v);
    if (16 < B / 8) v += lane_xor<16>(v);
    if (32 < B / 8) v += lane_xor<32>(v);
    return v;
}
template <int B>
__device__ __forceinline__ float block_allreduce_max(float v) {
    if (1 < B / 8) v = fmaxf(v, lane_xor<1>(v));
    if (2 < B / 8) v = fmaxf(v, lane_xor<2>(v));
    if (4 < B / 8) v = fmaxf(v, lane_xor<4>(v));
    if (8 < B / 8) v = fmaxf(v, lane_xor<8>(v));
    if (16 < B / 8) v = fmaxf(v, lane_xor<16>(v));
    if (32 < B / 8) v = fmaxf(v, lane_xor<32>(v));
    return v;
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

// The eight codes of two dwords as floats, q[r] = value of byte r (the conversions select the byte themselves).
__device__ __forceinline__ void decode8(u32x2 w, const Variant& var, float (&q)[8]) {
    const int lo = static_cast<int>(w.x), hi = static_cast<int>(w.y);
    if (var.format == 0) {
        q[0] = __builtin_amdgcn_cvt_f32_fp8(lo, 0); q[1] = __builtin_amdgcn_cvt_f32_fp8(lo, 1);
        q[2] = __builtin_amdgcn_cvt_f32_fp8(lo, 2); q[3] = __builtin_amdgcn_cvt_f32_fp8(lo, 3);
        q[4] = __builtin_amdgcn_cvt_f32_fp8(hi, 0); q[5] = __builtin_amdgcn_cvt_f32_fp8(hi, 1);
        q[6] = __builtin_amdgcn_cvt_f32_fp8(hi, 2); q[7] = __builtin_amdgcn_cvt_f32_fp8(hi, 3);
    } else if (var.format == 1) {
        q[0] = __builtin_amdgcn_cvt_f32_bf8(lo, 0); q[1] = __builtin_amdgcn_cvt_f32_bf8(lo, 1);
        q[2] = __builtin_amdgcn_cvt_f32_bf8(lo, 2); q[3] = __builtin_amdgcn_cvt_f32_bf8(lo, 3);
        q[4] = __builtin_amdgcn_cvt_f32_bf8(hi, 0); q[5] = __builtin_amdgcn_cvt_f32_bf8(hi, 1);
        q[6] = __builtin_amdgcn_cvt_f32_bf8(hi, 2); q[7] = __builtin_amdgcn_cvt_f32_bf8(hi, 3);
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            q[r] = static_cast<float>(static_cast<int8_t>((w.x >> (8 * r)) & 0xFF));
            q[4 + r] = static_cast<float>(static_cast<int8_t>((w.y >> (8 * r)) & 0xFF));
        }
    }
}

// Byte offset of block blk's codes in the payload buffer: blocks are B bytes apart in the split
// layout and B + 8 bytes apart (codes, then {alpha, s}) in the interleaved one.
template <int B>
__device__ __forceinline__ int64_t code_offset(int64_t blk, bool interleaved) {
    return blk * (interleaved ? B + 8 : B);
}

// Where a lane's eight elements sit: global block index and offset inside the block.
template <int B>
struct LaneSlot {
    int64_t blk;
    int pos;
    __device__ __forceinline__ LaneSlot(int64_t group, int lane)
        : blk(group * (kGroupElems / B) + lane / (B / 8)), pos(8 * (lane % (B / 8))) {}
};

// Eight codes of one lane as two dwords, byte r = code of q[r].
__device__ __forceinline__ u32x2 encode8(const float (&q)[8], const Variant& var) {
    u32x2 w;
    if (var.format == 0) {
        w.x = pack_e4m3x4(q[0], q[1], q[2], q[3]);
        w.y = pack_e4m3x4(q[4], q[5], q[6], q[7]);
    } else if (var.format == 1) {
        int lo = __builtin_amdgcn_cvt_pk_bf8_f32(q[0], q[1], 0, false);
        lo = __builtin_amdgcn_cvt_pk_bf8_f32(q[2], q[3], lo, true);
        int hi = __builtin_amdgcn_cvt_pk_bf8_f32(q[4], q[5], 0, false);
        hi = __builtin_amdgcn_cvt_pk_bf8_f32(q[6], q[7], hi, true);
        w.x = static_cast<uint32_t>(lo);
        w.y = static_cast<uint32_t>(hi);
    } else {
        uint32_t lo = 0, hi = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            lo |= static_cast<uint32_t>(encode_value(q[r], var)) << (8 * r);
            hi |= static_cast<uint32_t>(encode_value(q[4 + r], var)) << (8 * r);
        }
        w.x = lo;
        w.y = hi;
    }
    return w;
}

// Sender side of Algorithm 1 for the group whose elements are already in registers
// (v[r] = element 8 lane + r of the group, zeros past the end of the tensor).  Lanes whose block
// lies past the last block of the tensor take part in the exchanges and store nothing.
template <int B>
__device__ __forceinline__ void compress_group_butterfly(float (&v)[8], int lane, int64_t group, int64_t n_blocks_total,
                                                         float tau, float eps, uint8_t* __restrict__ payload,
                                                         f32x2* __restrict__ scales, bool interleaved, Variant var) {
    const LaneSlot<B> slot(group, lane);
    float alpha = 1.0f;
    if (var.rescale()) {
        float energy = 0.0f;
#pragma unroll
        for (int r = 0; r < 8; ++r) energy = __builtin_fmaf(v[r], v[r], energy);
        energy = block_allreduce_sum<B>(energy);                      // sum_j G_kj^2
        // Eq. ash_sigma, Eq. ash_alpha; an overflowing sum of squares is taken as the largest finite number (the codes do not
        // depend on alpha and the reconstruction only on s / alpha, so both stay right where alpha itself no longer is)
        alpha = tau * __builtin_amdgcn_rsqf(__builtin_fminf(energy * (1.0f / B), 0x1.fffffep+127f) + eps);
    }
    float norm = 1.0f, sign = 1.0f;
    if (var.rotate()) {
        sign = fwht_group<B>(v, lane);                                // W = sign * v = H G_k (unnormalised)
        norm = 1.0f / __builtin_sqrtf(static_cast<float>(B));
    }
    float wmax = 0.0f;
#pragma unroll
    for (int r = 0; r < 8; ++r) wmax = fmaxf(wmax, __builtin_fabsf(v[r]));
    wmax = block_allreduce_max<B>(wmax);
    const float qmax = var.qmax();
    // Z = alpha W / sqrt(B); with the post-rotation scale, s = max|Z| / Q_max (Eq. post_scale) and
    // Z / s = Q_max W / max|W| in exact arithmetic (zero blocks map to zero codes); without it s = 1
    // and Z itself is converted, saturating at +-Q_max.
    float s = 1.0f, to_code = alpha * norm;
    if (var.postscale()) {
        // an all-zero block stores s = 0 even where alpha is infinite (eps = 0)
        s = wmax > 0.0f ? (wmax * alpha * norm) * (1.0f / qmax) : 0.0f;
        to_code = wmax > 0.0f ? qmax * __builtin_amdgcn_rcpf(wmax) : 0.0f;
    }
    // Q_max / max|W| leaves fp32 when max|W| < 2^-118 (blocks of bf16 subnormals): take a power of two out first.
    if (var.postscale() && wmax > 0.0f && wmax < 0x1p-100f) {
        to_code = qmax * __builtin_amdgcn_rcpf(__builtin_ldexpf(wmax, 64));
#pragma unroll
        for (int r = 0; r < 8; ++r) v[r] = __builtin_ldexpf(v[r], 64);
    }
    if (slot.blk >= n_blocks_total) return;
    to_code *= sign;
    float q[8];
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        q[r] = v[r] * to_code;
        if (!var.postscale() || var.format == 2) q[r] = __builtin_amdgcn_fmed3f(q[r], -qmax, qmax);
    }
    uint8_t* dst = payload + code_offset<B>(slot.blk, interleaved);
    store_stream<true>(reinterpret_cast<u32x2*>(dst + slot.pos), encode8(q, var));
    if (slot.pos == 0) {
        if (interleaved) store_stream<true>(reinterpret_cast<f32x2*>(dst + B), f32x2{alpha, s});
        else store_stream<true>(&scales[slot.blk], f32x2{alpha, s});
    }
}

// The eight bf16 values of a 16-byte chunk as floats.
__device__ __forceinline__ void unpack_chunk(u32x4 w, float (&v)[8]) {
    v[0] = bf16_bits_to_f32(w.x & 0xFFFF); v[1] = bf16_bits_to_f32(w.x >> 16);
    v[2] = bf16_bits_to_f32(w.y & 0xFFFF); v[3] = bf16_bits_to_f32(w.y >> 16);
    v[4] = bf16_bits_to_f32(w.z & 0xFFFF); v[5] = bf16_bits_to_f32(w.z >> 16);
    v[6] = bf16_bits_to_f32(w.w & 0xFFFF); v[7] = bf16_bits_to_f32(w.w >> 16);
}

// Sender side of Algorithm 1: workgroup w of a tensor (one wave) handles its tile w.
template <int B>
__global__ __launch_bounds__(64) void compress_butterfly_kernel(CompressTable tab, int count, float tau, float eps,
                                                                bool interleaved, Variant var) {
    const int lane = threadIdx.x;
    int idx;
    int64_t tile;
    tab.locate(blockIdx.x, count, idx, tile);
    const u32x4* __restrict__ x = static_cast<const u32x4*>(tab.x(idx));
    const int64_t n = tab.n(idx);
    const int64_t n_blocks_total = (n + B - 1) / B;
    const int64_t first_elem = tile * (kGroupsPerTile * kGroupElems);
    u32x4 raw[kGroupsPerTile];
    if (first_elem + kGroupsPerTile * kGroupElems <= n) {
#pragma unroll
        for (int j = 0; j < kGroupsPerTile; ++j) raw[j] = load16<true>(&x[tile * 256 + 64 * j + lane]);
    } else {
#pragma unroll
        for (int j = 0; j < kGroupsPerTile; ++j) raw[j] = load_chunk_guarded(x, first_elem + 8 * (64 * j + lane), n);   // zero padding
    }
#pragma unroll
    for (int j = 0; j < kGroupsPerTile; ++j) {
        const int64_t group = tile * kGroupsPerTile + j;
        if (group * kGroupElems >= n) break;
        float v[8];
        unpack_chunk(raw[j], v);
        compress_group_butterfly<B>(v, lane, group, n_blocks_total, tau, eps, static_cast<uint8_t*>(tab.payload(idx)),
                                    static_cast<f32x2*>(tab.scales(idx)), interleaved, var);
    }
}

// Receiver side of Algorithm 1 plus the local reduction over k payloads for one group; the
// result (before the final rounding to bf16) is left in v.  The rotation is linear, so for
// k > 1 the codes are first combined with their block factors s / (alpha sqrt(B)) and rotated
// once; for k = 1 the raw codes are rotated (exact partial sums) and the factor is applied
// afterwards.  Lanes whose block lies past the end of the tensor read nothing and carry zeros.
template <int B>
__device__ __forceinline__ void decode_sum_group_butterfly(const DecodeTable& tab, int idx, int k, int64_t group, int lane,
                                                           int64_t n_blocks_total, float (&v)[8], bool interleaved,
                                                           Variant var) {
    const LaneSlot<B> slot(group, lane);
    const bool live = slot.blk < n_blocks_total;
    const float inv_root_b = var.rotate() ? 1.0f / __builtin_sqrtf(static_cast<float>(B)) : 1.0f;
#pragma unroll
    for (int r = 0; r < 8; ++r) v[r] = 0.0f;
    float single = 1.0f;
    // Four payloads at a time, all their loads issued before the first is used.
    for (int i0 = 0; i0 < k; i0 += 4) {
        u32x2 w8[4];
        f32x2 sc[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            w8[j] = u32x2{0, 0};
            sc[j] = f32x2{1.0f, 0.0f};
            if (live && i0 + j < k) {
                const uint8_t* codes = static_cast<const uint8_t*>(tab.payload(idx, k, i0 + j)) + code_offset<B>(slot.blk, interleaved);
                sc[j] = interleaved ? *reinterpret_cast<const f32x2*>(codes + B)
                                    : static_cast<const f32x2*>(tab.scales(idx, k, i0 + j))[slot.blk];
                w8[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(codes + slot.pos));
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (i0 + j < k) {
                const float factor = sc[j].y * __builtin_amdgcn_rcpf(sc[j].x) * inv_root_b;   // s / (alpha sqrt(B))
                const float w = (k == 1) ? 1.0f : factor;
                single = factor;
                float q[8];
                decode8(w8[j], var, q);
#pragma unroll
                for (int r = 0; r < 8; ++r) v[r] = __builtin_fmaf(q[r], w, v[r]);
            }
        }
    }
    const float sign = var.rotate() ? fwht_group<B>(v, lane) : 1.0f;
    const float post = (k == 1) ? single * sign : sign;
#pragma unroll
    for (int r = 0; r < 8; ++r) v[r] *= post;
}

// Receiver side of Algorithm 1 and the local reduction: workgroup w of a tensor (one wave) handles its tile w.
template <int B>
__global__ __launch_bounds__(64) void decompress_sum_butterfly_kernel(DecodeTable tab, int count, int k, bool interleaved, Variant var) {
    const int lane = threadIdx.x;
    int idx;
    int64_t tile;
    tab.locate(blockIdx.x, count, idx, tile);
    const int64_t n = tab.n(idx);
    const int64_t n_blocks_total = (n + B - 1) / B;
    uint16_t* __restrict__ out = static_cast<uint16_t*>(tab.output(idx));
#pragma unroll
    for (int j = 0; j < kGroupsPerTile; ++j) {
        const int64_t g = tile * kGroupsPerTile + j;
        if (g * kGroupElems >= n) break;
        float v[8];
        decode_sum_group_butterfly<B>(tab, idx, k, g, lane, n_blocks_total, v, interleaved, var);
        const int64_t first = g * kGroupElems + 8 * lane;
        if (first + 8 <= n) {
            u32x4 w;
            w.x = pack_bf16x2(v[0], v[1]); w.y = pack_bf16x2(v[2], v[3]);
            w.z = pack_bf16x2(v[4], v[5]); w.w = pack_bf16x2(v[6], v[7]);
            store_stream<true>(reinterpret_cast<u32x4*>(out + first), w);
        } else {
#pragma unroll
            for (int r = 0; r < 8; ++r)
                if (first + r < n) out[first + r] = static_cast<uint16_t>(pack_bf16x2(v[r], 0.0f) & 0xFFFF);
        }
    }
}

// decompress_sum followed by compress of the bf16-rounded sum, group by group, without the
// bf16 tensor leaving the registers.
template <int B>
__global__ __launch_bounds__(64) void decompress_sum_compress_butterfly_kernel(DecodeTable tab, int count, int k, float tau, float eps,
                                                                               bool interleaved, Variant var) {
    const int lane = threadIdx.x;
    int idx;
    int64_t tile;
    tab.locate(blockIdx.x, count, idx, tile);
    const int64_t n = tab.n(idx);
    const int64_t n_blocks_total = (n + B - 1) / B;
#pragma unroll
    for (int j = 0; j < kGroupsPerTile; ++j) {
        const int64_t g = tile * kGroupsPerTile + j;
        if (g * kGroupElems >= n) break;
        float v[8];
        decode_sum_group_butterfly<B>(tab, idx, k, g, lane, n_blocks_total, v, interleaved, var);
        const int64_t first = g * kGroupElems + 8 * lane;
#pragma unroll
        for (int r = 0; r < 8; ++r)
            v[r] = first + r < n ? bf16_bits_to_f32(pack_bf16x2(v[r], 0.0f) & 0xFFFF) : 0.0f;
        compress_group_butterfly<B>(v, lane, g, n_blocks_total, tau, eps, static_cast<uint8_t*>(tab.payload_output(idx)),
                                    static_cast<f32x2*>(tab.scales_output(idx)), interleaved, var);
    }
}

}  // namespace taco
