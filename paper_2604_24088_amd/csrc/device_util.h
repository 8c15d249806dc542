// Device-side helpers shared by the gfx950 kernels: type punning, bf16 / FP8 conversion
// instructions, DPP lane exchanges inside a 16-lane row, wave-local LDS ordering.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace taco {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));   // one {alpha, s} record
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte load / store / LDS slot
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr float kQmax = 448.0f;  // largest finite E4M3 value (Q_max of Eq. post_scale)

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) {
    return __builtin_bit_cast(float, bits16 << 16);
}

// binary32 -> bf16, round to nearest even (v_cvt_pk_bf16_f32 on gfx950).
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 v2 __attribute__((ext_vector_type(2)));
    v2 p;
    p[0] = static_cast<__bf16>(lo);
    p[1] = static_cast<__bf16>(hi);
    return __builtin_bit_cast(uint32_t, p);
}

// Four floats -> four E4M3 codes in one dword, byte i = code of v_i (round to nearest even).
__device__ __forceinline__ uint32_t pack_e4m3x4(float v0, float v1, float v2, float v3) {
    int w = __builtin_amdgcn_cvt_pk_fp8_f32(v0, v1, 0, false);
    w = __builtin_amdgcn_cvt_pk_fp8_f32(v2, v3, w, true);
    return static_cast<uint32_t>(w);
}

// The same for E5M2 codes (the format ablation's other 8-bit float).
__device__ __forceinline__ uint32_t pack_e5m2x4(float v0, float v1, float v2, float v3) {
    int w = __builtin_amdgcn_cvt_pk_bf8_f32(v0, v1, 0, false);
    w = __builtin_amdgcn_cvt_pk_bf8_f32(v2, v3, w, true);
    return static_cast<uint32_t>(w);
}

// Four floats, each times f, -> four INT8 codes in one dword (round to nearest, ties to even).
// fma(v, f, 1.5 * 2^23) rounds the EXACT product to an integer in one step (the sum lies in
// [2^23, 2^24), where fp32 numbers are the integers) and leaves that integer, in two's complement,
// in the low bits of the result; |v f| <= 127 (1 + 2^-22) by construction, so no clamp is needed.
__device__ __forceinline__ uint32_t pack_int8x4_scaled(float v0, float v1, float v2, float v3, float f) {
    constexpr float kMagic = 12582912.0f;
    const uint32_t b0 = __builtin_bit_cast(uint32_t, __builtin_fmaf(v0, f, kMagic));
    const uint32_t b1 = __builtin_bit_cast(uint32_t, __builtin_fmaf(v1, f, kMagic));
    const uint32_t b2 = __builtin_bit_cast(uint32_t, __builtin_fmaf(v2, f, kMagic));
    const uint32_t b3 = __builtin_bit_cast(uint32_t, __builtin_fmaf(v3, f, kMagic));
    const uint32_t lo = __builtin_amdgcn_perm(b1, b0, 0x0c0c0400u);    // bytes: b0.0, b1.0, 0, 0
    const uint32_t hi = __builtin_amdgcn_perm(b3, b2, 0x04000c0cu);    // bytes: 0, 0, b2.0, b3.0
    return lo | hi;
}

// Code book of the matrix-core kernels: 0 = E4M3 (the method), 1 = E5M2, 2 = INT8 (format ablation).
// Byte i of the result = code of v_i * f.
template <int kFormat>
__device__ __forceinline__ uint32_t pack_codes4(float v0, float v1, float v2, float v3, float f) {
    if (kFormat == 0) return pack_e4m3x4(v0 * f, v1 * f, v2 * f, v3 * f);
    if (kFormat == 1) return pack_e5m2x4(v0 * f, v1 * f, v2 * f, v3 * f);
    return pack_int8x4_scaled(v0, v1, v2, v3, f);
}
// The same for values that may lie outside the code book's range (the variants without the post-rotation
// scale): v_i * f is clamped to +-Q_max first.
template <int kFormat>
__device__ __forceinline__ uint32_t pack_codes4_clamped(float v0, float v1, float v2, float v3, float f) {
    constexpr float kQ = kFormat == 0 ? 448.0f : kFormat == 1 ? 57344.0f : 127.0f;
    return pack_codes4<kFormat>(__builtin_amdgcn_fmed3f(v0 * f, -kQ, kQ), __builtin_amdgcn_fmed3f(v1 * f, -kQ, kQ),
                                __builtin_amdgcn_fmed3f(v2 * f, -kQ, kQ), __builtin_amdgcn_fmed3f(v3 * f, -kQ, kQ), 1.0f);
}
template <int kFormat>
__device__ __forceinline__ constexpr float format_qmax() { return kFormat == 0 ? 448.0f : kFormat == 1 ? 57344.0f : 127.0f; }

// Sum of squares of the two bf16 halves of a dword, added to acc (v_dot2c_f32_bf16).
// The dword is taken BY VALUE: bit-casting a vector-element lvalue directly reads element 0.
__device__ __forceinline__ float dot2_self_bf16(uint32_t pair, float acc) {
    const bf16x2 p = __builtin_bit_cast(bf16x2, pair);
    return __builtin_amdgcn_fdot2_f32_bf16(p, p, acc, false);
}

// Streaming (non-temporal) global accesses: data that is touched once should not displace
// anything in the caches.  kStream = false gives the ordinary access.
template <bool kStream>
__device__ __forceinline__ u32x4 load16(const u32x4* p) {
    return kStream ? __builtin_nontemporal_load(p) : *p;
}
template <bool kStream, typename T>
__device__ __forceinline__ void store_stream(T* p, T v) {
    if (kStream) __builtin_nontemporal_store(v, p); else *p = v;
}

// One 16-byte chunk (8 bf16) whose first element is e0, from a tensor of n elements at x: the part of
// it that exists, zeros for the rest.  Only the wave that owns a partial last tile comes here.
__device__ __forceinline__ u32x4 load_chunk_guarded(const u32x4* __restrict__ x, int64_t e0, int64_t n) {
    if (e0 + 8 <= n) return load16<true>(&x[e0 >> 3]);
    const uint16_t* xe = reinterpret_cast<const uint16_t*>(x);
    uint32_t w[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int r = 0; r < 8; ++r)
        if (e0 + r < n) w[r >> 1] |= static_cast<uint32_t>(xe[e0 + r]) << (16 * (r & 1));
    return u32x4{w[0], w[1], w[2], w[3]};
}

__device__ __forceinline__ int parity32(uint32_t v) { return __builtin_popcount(v) & 1; }

// ---- DPP: data movement inside a row of 16 lanes --------------------------------------

template <int kCtrl>
__device__ __forceinline__ float dpp_f32(float v) {
    int r = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), kCtrl, 0xF, 0xF, true);
    return __builtin_bit_cast(float, r);
}

template <int kCtrl>
__device__ __forceinline__ uint32_t dpp_u32(uint32_t v) {
    return static_cast<uint32_t>(__builtin_amdgcn_update_dpp(0, static_cast<int>(v), kCtrl, 0xF, 0xF, true));
}

constexpr int kDppRowRor(int n) { return 0x120 + n; }                  // rotate right by n in the row
constexpr int kDppQuadBcast(int q) { return q | (q << 2) | (q << 4) | (q << 6); }  // lane q of each quad

// The value held by lane (lane ^ kMask).  Masks inside a row of 16 lanes are DPP moves (quad
// permutes for 1 and 2; for 4 the mirror of each half row, lane ^ 7, followed by the reversal of
// each quad, lane ^ 3; for 8 the rotation by half a row); 16 and 32 go through the LDS crossbar.
template <int kMask>
__device__ __forceinline__ float lane_xor(float v) {
    static_assert(kMask == 1 || kMask == 2 || kMask == 4 || kMask == 8 || kMask == 16 || kMask == 32, "one lane bit");
    if (kMask == 1) return dpp_f32<0xB1>(v);                      // quad_perm [1,0,3,2]
    if (kMask == 2) return dpp_f32<0x4E>(v);                      // quad_perm [2,3,0,1]
    if (kMask == 4) return dpp_f32<0x1B>(dpp_f32<0x141>(v));      // row_half_mirror, then quad_perm [3,2,1,0]
    if (kMask == 8) return dpp_f32<kDppRowRor(8)>(v);
    return __shfl_xor(v, kMask, 64);
}

// Orders one wave's LDS accesses: what its lanes wrote before is visible to what they read after.
// LDS instructions of a wave execute in issue order, so no instruction is needed: the fences only
// stop the compiler from moving LDS accesses across this point.  Every wave of the matrix-core
// kernels works in an LDS region of its own, so no workgroup barrier is ever needed (and waves of
// one workgroup may run different numbers of loop iterations).
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

}  // namespace taco
