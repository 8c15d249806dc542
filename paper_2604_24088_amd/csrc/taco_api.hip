// Host side of the C ABI declared in include/taco.h: argument checks, kernel choice,
// launch geometry.  No device memory is allocated and nothing is synchronised here.

#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdint>
#include <type_traits>

#include "../../include/taco.h"
#include "butterfly_kernels.h"
#include "device_util.h"
#include "mfma_kernels.h"

namespace {

constexpr int64_t kMaxElems = int64_t(1) << 40;

bool block_ok(int32_t b) { return b == 32 || b == 64 || b == 128 || b == 256 || b == 512; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Compute-unit count of the current device, queried once per device; safe to call from several
// threads (the worst case is two threads asking the runtime the same question).
int device_cus() {
    constexpr int kMaxDevices = 64;
    static std::atomic<int> cache[kMaxDevices];      // zero-initialised: 0 = not asked yet
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
    int v = cache[dev].load(std::memory_order_relaxed);
    if (v > 0) return v;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
    cache[dev].store(v, std::memory_order_relaxed);
    return v;
}

// The matrix-core kernels implement the method itself and the variants that keep its structure
// (rotation and post-rotation scale on, an 8-bit float code book): the full method and the
// "standard Hadamard" ablation (no adaptive rescaling), in E4M3 or E5M2.  Everything else runs on
// the butterfly kernels.
bool mfma_capable(const taco_params* p) {
    return (p->mode == TACO_MODE_FULL || p->mode == (TACO_MODE_ROTATE | TACO_MODE_POSTSCALE)) &&
           (p->format == TACO_FORMAT_E4M3 || p->format == TACO_FORMAT_E5M2);
}

int check_common(int64_t rows, int64_t cols, const taco_params* p, int64_t* n_out) {
    if (!p) return TACO_ERR_NULL;
    if (rows <= 0 || cols <= 0) return TACO_ERR_SHAPE;
    if (rows > kMaxElems || cols > kMaxElems || rows > kMaxElems / cols) return TACO_ERR_SHAPE;
    if (!block_ok(p->block)) return TACO_ERR_BLOCK;
    if (p->format != TACO_FORMAT_E4M3 && p->format != TACO_FORMAT_E5M2 && p->format != TACO_FORMAT_INT8) return TACO_ERR_FORMAT;
    if (p->mode < 0 || p->mode > TACO_MODE_FULL) return TACO_ERR_MODE;
    if (p->impl != TACO_IMPL_AUTO && p->impl != TACO_IMPL_BUTTERFLY && p->impl != TACO_IMPL_MFMA) return TACO_ERR_IMPL;
    if (p->layout != TACO_LAYOUT_SPLIT && p->layout != TACO_LAYOUT_INTERLEAVED) return TACO_ERR_LAYOUT;
    if (p->impl == TACO_IMPL_MFMA && !mfma_capable(p)) return TACO_ERR_IMPL;
    *n_out = rows * cols;
    return TACO_OK;
}

bool use_mfma(const taco_params* p) { return p->impl != TACO_IMPL_BUTTERFLY && mfma_capable(p); }

taco::Variant variant_of(const taco_params* p) { return taco::Variant{p->mode, p->format}; }

// Grid of the butterfly kernels: one single-wave workgroup per work item (one-shot waves, as in the
// matrix-core kernels) up to waves_per_cu per compute unit, a stride loop beyond that.
int grid_for(int64_t work_items, int waves_per_cu) {
    int64_t cap = static_cast<int64_t>(device_cus()) * waves_per_cu;
    int64_t g = work_items < cap ? work_items : cap;
    return static_cast<int>(g < 1 ? 1 : g);
}

template <typename F>
int dispatch_block(int32_t block, F&& f) {
    switch (block) {
        case 32: f(std::integral_constant<int, 32>{}); return TACO_OK;
        case 64: f(std::integral_constant<int, 64>{}); return TACO_OK;
        case 128: f(std::integral_constant<int, 128>{}); return TACO_OK;
        case 256: f(std::integral_constant<int, 256>{}); return TACO_OK;
        case 512: f(std::integral_constant<int, 512>{}); return TACO_OK;
        default: return TACO_ERR_BLOCK;
    }
}

int launch_status() { return hipGetLastError() == hipSuccess ? TACO_OK : TACO_ERR_LAUNCH; }

bool params_ok_for_compress(const taco_params* p) {
    return p->tau > 0.0f && p->eps >= 0.0f && std::isfinite(p->tau) && std::isfinite(p->eps);
}

// Calls f(kRB, kSub, kInterleaved, kFormat) with the four as compile-time constants.
template <typename F>
void dispatch_shape(int block, bool interleaved, int format, F&& f) {
    auto with_layout = [&](auto rb, auto sub) {
        using std::integral_constant;
        if (format == TACO_FORMAT_E5M2) {
            if (interleaved) f(rb, sub, std::true_type{}, integral_constant<int, 1>{});
            else f(rb, sub, std::false_type{}, integral_constant<int, 1>{});
        } else {
            if (interleaved) f(rb, sub, std::true_type{}, integral_constant<int, 0>{});
            else f(rb, sub, std::false_type{}, integral_constant<int, 0>{});
        }
    };
    using std::integral_constant;
    switch (block) {
        case 32: with_layout(integral_constant<int, 1>{}, integral_constant<int, 4>{}); break;
        case 64: with_layout(integral_constant<int, 1>{}, integral_constant<int, 2>{}); break;
        case 128: with_layout(integral_constant<int, 1>{}, integral_constant<int, 1>{}); break;
        case 256: with_layout(integral_constant<int, 2>{}, integral_constant<int, 1>{}); break;
        default: with_layout(integral_constant<int, 4>{}, integral_constant<int, 1>{}); break;
    }
}

// Fills the kernel-side table from the caller's host arrays.  In the interleaved layout the
// scales live inside the payload and `scales` (the array or its entries) may be NULL.
int fill_table(const void* const* payloads, const void* const* scales, int k, bool interleaved, taco::PayloadTable* tab) {
    if (!payloads || (!interleaved && !scales)) return TACO_ERR_NULL;
    for (int i = 0; i < k; ++i) {
        if (!payloads[i] || (!interleaved && !scales[i])) return TACO_ERR_NULL;
        if (!aligned16(payloads[i]) || (!interleaved && !aligned16(scales[i]))) return TACO_ERR_ALIGN;
        tab->payload[i] = payloads[i];
        tab->scales[i] = interleaved ? nullptr : scales[i];
    }
    return TACO_OK;
}

// Decode (and optionally re-compress) whole tiles on the matrix cores, the rest on the butterfly kernel.
int launch_decode(const taco::PayloadTable& tab, int k, int64_t n, const taco_params* p, bool recompress,
                  void* out_bf16, void* payload_out, void* scales_out, hipStream_t st) {
    const int B = p->block;
    const bool il = p->layout == TACO_LAYOUT_INTERLEAVED;
    int64_t first_group = 0;       // groups of 512 elements: what one wave of the butterfly kernels handles
    if (use_mfma(p)) {
        const int64_t n_tiles = n / taco::kTileElems;
        if (n_tiles > 0) {
            // Launch shape, measured on MI355X (1..16 tiles per wave, rings of 2..8 items, 1..8 waves
            // per workgroup tried, all block sizes and both layouts): a ring of four (tile, payload)
            // items in flight; up to five payloads, and for the recompress form, two output tiles per
            // wave and one wave per workgroup; from six payloads on, one tile per wave and two waves
            // per workgroup (3-10 % faster at k = 8..16, 5-10 % slower at k <= 4).
            const bool wide = !recompress && k >= 6;
            // The recompress form at B = 32 (its heaviest epilogue) is 6-9 % faster with one tile per wave.
            const bool single = recompress && B == 32;
            const int tiles_per_wave = (wide || single) ? 1 : 2;
            const int64_t tiles_per_group = single ? 1 : 2;      // 1 wave x 2 tiles, 2 waves x 1 tile, or 1 x 1
            const unsigned groups = static_cast<unsigned>((n_tiles + tiles_per_group - 1) / tiles_per_group);
            const bool rescale = (p->mode & TACO_MODE_RESCALE) != 0;
            dispatch_shape(B, il, p->format, [&](auto rb, auto sub, auto layout, auto fmt) {
                constexpr int kRB = decltype(rb)::value, kSub = decltype(sub)::value, kFmt = decltype(fmt)::value;
                constexpr bool kIl = decltype(layout)::value;
                if (recompress)
                    hipLaunchKernelGGL((taco::decompress_sum_mfma_kernel<kRB, kSub, 4, kIl, true, 1, kFmt>), dim3(groups), dim3(64),
                                       0, st, tab, k, n_tiles, tiles_per_wave, static_cast<taco::u32x4*>(nullptr), p->tau, p->eps,
                                       static_cast<taco::u32x2*>(payload_out), static_cast<taco::f32x2*>(scales_out), rescale);
                else if (wide)
                    hipLaunchKernelGGL((taco::decompress_sum_mfma_kernel<kRB, kSub, 4, kIl, false, 2, kFmt>), dim3(groups), dim3(128),
                                       0, st, tab, k, n_tiles, tiles_per_wave, static_cast<taco::u32x4*>(out_bf16), 0.0f, 0.0f,
                                       static_cast<taco::u32x2*>(nullptr), static_cast<taco::f32x2*>(nullptr), true);
                else
                    hipLaunchKernelGGL((taco::decompress_sum_mfma_kernel<kRB, kSub, 4, kIl, false, 1, kFmt>), dim3(groups), dim3(64),
                                       0, st, tab, k, n_tiles, tiles_per_wave, static_cast<taco::u32x4*>(out_bf16), 0.0f, 0.0f,
                                       static_cast<taco::u32x2*>(nullptr), static_cast<taco::f32x2*>(nullptr), true);
            });
            if (int rc = launch_status()) return rc;
        }
        first_group = n_tiles * (taco::kTileElems / taco::kGroupElems);
    }
    const int64_t rest = (n - first_group * taco::kGroupElems + taco::kGroupElems - 1) / taco::kGroupElems;
    if (rest > 0) {
        const float tau = p->tau, eps = p->eps;
        int rc = dispatch_block(B, [&](auto bc) {
            constexpr int kB = decltype(bc)::value;
            if (recompress)
                hipLaunchKernelGGL(taco::decompress_sum_compress_butterfly_kernel<kB>, dim3(grid_for(rest, 16384)), dim3(64), 0, st,
                                   tab, k, n, first_group, rest, tau, eps, static_cast<uint8_t*>(payload_out),
                                   static_cast<float2*>(scales_out), il, variant_of(p));
            else
                hipLaunchKernelGGL(taco::decompress_sum_butterfly_kernel<kB>, dim3(grid_for(rest, 16384)), dim3(64), 0, st,
                                   tab, k, n, first_group, rest, static_cast<uint16_t*>(out_bf16), il, variant_of(p));
        });
        if (rc) return rc;
        if (int rc2 = launch_status()) return rc2;
    }
    return TACO_OK;
}

}  // namespace

extern "C" {

void taco_default_params(taco_params* p) {
    if (!p) return;
    p->block = 128;
    p->tau = 1.0f;
    p->eps = 1e-12f;
    p->format = TACO_FORMAT_E4M3;
    p->impl = TACO_IMPL_AUTO;
    p->layout = TACO_LAYOUT_SPLIT;
    p->mode = TACO_MODE_FULL;
}

size_t taco_payload_bytes(int64_t n, int32_t block) {
    if (n <= 0 || n > kMaxElems || !block_ok(block)) return 0;
    return static_cast<size_t>((n + block - 1) / block) * static_cast<size_t>(block);
}

size_t taco_scales_bytes(int64_t n, int32_t block) {
    if (n <= 0 || n > kMaxElems || !block_ok(block)) return 0;
    return static_cast<size_t>((n + block - 1) / block) * 8u;
}

int taco_compress(const void* x_bf16, int64_t rows, int64_t cols, const taco_params* p,
                  void* payload, void* scales, void* stream) {
    if (!x_bf16 || !payload) return TACO_ERR_NULL;
    int64_t n = 0;
    if (int rc = check_common(rows, cols, p, &n)) return rc;
    const bool il = p->layout == TACO_LAYOUT_INTERLEAVED;
    if (!il && !scales) return TACO_ERR_NULL;
    if (!params_ok_for_compress(p)) return TACO_ERR_PARAM;
    if (!aligned16(x_bf16) || !aligned16(payload) || (!il && !aligned16(scales))) return TACO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int B = p->block;
    int64_t first_group = 0;       // groups of 512 elements: what one wave of the butterfly kernels handles
    if (use_mfma(p)) {
        const int64_t n_tiles = n / taco::kTileElems;
        if (n_tiles > 0) {
            // One tile per wave, one wave per workgroup: measured best on MI355X at every block size
            // and in both layouts (2 tiles per wave cost 4-5 % on the largest tensors, 4 more).
            const unsigned waves = static_cast<unsigned>(n_tiles);
            const auto* xin = static_cast<const taco::u32x4*>(x_bf16);
            auto* pout = static_cast<taco::u32x2*>(payload);
            auto* sout = static_cast<taco::f32x2*>(scales);
            const bool rescale = (p->mode & TACO_MODE_RESCALE) != 0;
            dispatch_shape(B, il, p->format, [&](auto rb, auto sub, auto layout, auto fmt) {
                constexpr int kRB = decltype(rb)::value, kSub = decltype(sub)::value, kFmt = decltype(fmt)::value;
                constexpr bool kIl = decltype(layout)::value;
                hipLaunchKernelGGL((taco::compress_mfma_kernel<kRB, kSub, 1, kIl, kFmt>), dim3(waves), dim3(64), 0, st,
                                   xin, n_tiles, p->tau, p->eps, pout, sout, rescale);
            });
            if (int rc = launch_status()) return rc;
        }
        first_group = n_tiles * (taco::kTileElems / taco::kGroupElems);
    }
    const int64_t rest = (n - first_group * taco::kGroupElems + taco::kGroupElems - 1) / taco::kGroupElems;
    if (rest > 0) {
        const float tau = p->tau, eps = p->eps;
        int rc = dispatch_block(B, [&](auto bc) {
            constexpr int kB = decltype(bc)::value;
            hipLaunchKernelGGL(taco::compress_butterfly_kernel<kB>, dim3(grid_for(rest, 16384)), dim3(64), 0, st,
                               static_cast<const uint16_t*>(x_bf16), n, first_group, rest, tau, eps,
                               static_cast<uint8_t*>(payload), static_cast<float2*>(scales), il, variant_of(p));
        });
        if (rc) return rc;
        if (int rc2 = launch_status()) return rc2;
    }
    return TACO_OK;
}

int taco_decompress_sum(const void* const* payloads, const void* const* scales, int32_t k,
                        int64_t rows, int64_t cols, const taco_params* p, void* out_bf16,
                        void* stream) {
    if (!out_bf16) return TACO_ERR_NULL;
    if (k < 1 || k > TACO_MAX_K) return TACO_ERR_K;
    int64_t n = 0;
    if (int rc = check_common(rows, cols, p, &n)) return rc;
    taco::PayloadTable tab{};
    if (int rc = fill_table(payloads, scales, k, p->layout == TACO_LAYOUT_INTERLEAVED, &tab)) return rc;
    if (!aligned16(out_bf16)) return TACO_ERR_ALIGN;
    return launch_decode(tab, k, n, p, false, out_bf16, nullptr, nullptr, static_cast<hipStream_t>(stream));
}

int taco_decompress_sum_compress(const void* const* payloads, const void* const* scales, int32_t k,
                                 int64_t rows, int64_t cols, const taco_params* p, void* payload_out,
                                 void* scales_out, void* stream) {
    if (!payload_out) return TACO_ERR_NULL;
    if (k < 1 || k > TACO_MAX_K) return TACO_ERR_K;
    int64_t n = 0;
    if (int rc = check_common(rows, cols, p, &n)) return rc;
    const bool il = p->layout == TACO_LAYOUT_INTERLEAVED;
    if (!il && !scales_out) return TACO_ERR_NULL;
    if (!params_ok_for_compress(p)) return TACO_ERR_PARAM;
    taco::PayloadTable tab{};
    if (int rc = fill_table(payloads, scales, k, il, &tab)) return rc;
    if (!aligned16(payload_out) || (!il && !aligned16(scales_out))) return TACO_ERR_ALIGN;
    return launch_decode(tab, k, n, p, true, nullptr, payload_out, scales_out, static_cast<hipStream_t>(stream));
}

int taco_decompress(const void* payload, const void* scales, int64_t rows, int64_t cols,
                    const taco_params* p, void* out_bf16, void* stream) {
    const void* pl[1] = {payload};
    const void* sc[1] = {scales};
    return taco_decompress_sum(pl, sc, 1, rows, cols, p, out_bf16, stream);
}

int taco_debug_cvt_e4m3(const void* in_f32, int64_t n, void* out_codes, void* stream) {
    if (!in_f32 || !out_codes) return TACO_ERR_NULL;
    if (n <= 0 || n > kMaxElems) return TACO_ERR_SHAPE;
    const int threads = 256;
    const int64_t blocks = (n + threads - 1) / threads;
    if (blocks > 0x7fffffff) return TACO_ERR_SHAPE;
    hipLaunchKernelGGL(taco::cvt_e4m3_kernel, dim3(static_cast<unsigned>(blocks)), dim3(threads), 0,
                       static_cast<hipStream_t>(stream), static_cast<const float*>(in_f32), n,
                       static_cast<uint8_t*>(out_codes));
    return launch_status();
}

int taco_debug_copy(const void* src, void* dst, int64_t bytes, void* stream) {
    if (!src || !dst) return TACO_ERR_NULL;
    if (bytes <= 0 || (bytes & 15) != 0) return TACO_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(dst)) return TACO_ERR_ALIGN;
    const int64_t n16 = bytes / 16;
    const int64_t want = (n16 + 255) / 256;
    const int64_t cap = static_cast<int64_t>(device_cus()) * 32;
    hipLaunchKernelGGL(taco::copy_kernel, dim3(static_cast<unsigned>(want < cap ? want : cap)), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const taco::u32x4*>(src),
                       static_cast<taco::u32x4*>(dst), n16);
    return launch_status();
}

int taco_debug_traffic(const void* const* srcs, int32_t k, int32_t src_chunks, void* dst,
                       int32_t dst_chunks, int64_t n_tiles, void* stream) {
    if (!srcs || !dst) return TACO_ERR_NULL;
    if (k < 1 || k > TACO_MAX_K) return TACO_ERR_K;
    if (src_chunks < 1 || src_chunks > 256 || dst_chunks < 1 || dst_chunks > 256) return TACO_ERR_SHAPE;
    if (n_tiles < 1 || n_tiles > kMaxElems / taco::kTileElems) return TACO_ERR_SHAPE;
    taco::PayloadTable tab{};
    for (int i = 0; i < k; ++i) {
        if (!srcs[i]) return TACO_ERR_NULL;
        if (!aligned16(srcs[i])) return TACO_ERR_ALIGN;
        tab.payload[i] = srcs[i];
    }
    if (!aligned16(dst)) return TACO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // The launch shapes of the kernels it stands in for: two waves per workgroup from six sources on.
    if (k >= 6)
        hipLaunchKernelGGL(taco::traffic_kernel<2>, dim3(static_cast<unsigned>((n_tiles + 1) / 2)), dim3(128), 0, st,
                           tab, k, src_chunks, static_cast<taco::u32x4*>(dst), dst_chunks, n_tiles);
    else
        hipLaunchKernelGGL(taco::traffic_kernel<1>, dim3(static_cast<unsigned>(n_tiles)), dim3(64), 0, st,
                           tab, k, src_chunks, static_cast<taco::u32x4*>(dst), dst_chunks, n_tiles);
    return launch_status();
}

const char* taco_strerror(int status) {
    switch (status) {
        case TACO_OK: return "ok";
        case TACO_ERR_NULL: return "null pointer";
        case TACO_ERR_SHAPE: return "bad shape: rows and cols must be positive and rows*cols at most 2^40";
        case TACO_ERR_BLOCK: return "bad block size: must be 32, 64, 128, 256 or 512";
        case TACO_ERR_ALIGN: return "data pointer is not 16-byte aligned";
        case TACO_ERR_K: return "k must be between 1 and 16";
        case TACO_ERR_FORMAT: return "bad format: must be E4M3, E5M2 or INT8";
        case TACO_ERR_LAUNCH: return "kernel launch failed";
        case TACO_ERR_IMPL: return "bad kernel selection (the matrix-core kernels cover modes 7 and 6 in E4M3 or E5M2)";
        case TACO_ERR_PARAM: return "bad parameter: tau must be positive and eps non-negative, both finite";
        case TACO_ERR_LAYOUT: return "bad layout: must be split or interleaved";
        case TACO_ERR_MODE: return "bad mode: must be a combination of the three TACO_MODE_* bits";
        default: return "unknown status";
    }
}

const char* taco_version(void) { return "0.3"; }

}  // extern "C"
