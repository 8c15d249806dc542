// Host side of the C ABI declared in include/taco.h: argument checks, kernel choice,
// launch geometry.  No device memory is allocated and nothing is synchronised here.

#include <hip/hip_runtime.h>

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

struct DeviceInfo {
    int cus = 0;
};

// Compute-unit count of the current device (queried once per process and device id).
int device_cus() {
    static int cached_dev = -1;
    static int cached_cus = 0;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (dev != cached_dev) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
        cached_cus = v;
        cached_dev = dev;
    }
    return cached_cus;
}

int check_common(int64_t rows, int64_t cols, const taco_params* p, int64_t* n_out) {
    if (!p) return TACO_ERR_NULL;
    if (rows <= 0 || cols <= 0) return TACO_ERR_SHAPE;
    if (rows > kMaxElems || cols > kMaxElems || rows > kMaxElems / cols) return TACO_ERR_SHAPE;
    if (!block_ok(p->block)) return TACO_ERR_BLOCK;
    if (p->format != TACO_FORMAT_E4M3) return TACO_ERR_FORMAT;
    if (p->impl != TACO_IMPL_AUTO && p->impl != TACO_IMPL_BUTTERFLY && p->impl != TACO_IMPL_MFMA) return TACO_ERR_IMPL;
    *n_out = rows * cols;
    return TACO_OK;
}

bool use_mfma(const taco_params* p) { return p->impl != TACO_IMPL_BUTTERFLY; }

// Persistent grids: enough single-wave workgroups to fill every SIMD several times over.
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

}  // namespace

extern "C" {

void taco_default_params(taco_params* p) {
    if (!p) return;
    p->block = 128;
    p->tau = 1.0f;
    p->eps = 1e-12f;
    p->format = TACO_FORMAT_E4M3;
    p->impl = TACO_IMPL_AUTO;
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
    if (!x_bf16 || !payload || !scales) return TACO_ERR_NULL;
    int64_t n = 0;
    if (int rc = check_common(rows, cols, p, &n)) return rc;
    if (!(p->tau > 0.0f) || !(p->eps >= 0.0f) || !std::isfinite(p->tau) || !std::isfinite(p->eps)) return TACO_ERR_PARAM;
    if (!aligned16(x_bf16) || !aligned16(payload) || !aligned16(scales)) return TACO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int B = p->block;
    const int64_t n_blocks = (n + B - 1) / B;
    int64_t first_block = 0;
    if (use_mfma(p)) {
        const int64_t n_tiles = n / taco::kTileElems;
        if (n_tiles > 0) {
            // Tiles per wave, measured on MI355X: 2 wins on the largest tensors (98 k tiles), 1 below
            // (finer tail, more waves to fill 256 compute units); 4 loses everywhere.
            const bool two = n_tiles >= 65536;
            const unsigned waves = static_cast<unsigned>(two ? (n_tiles + 1) / 2 : n_tiles);
            const auto* xin = static_cast<const taco::u32x4*>(x_bf16);
            auto* pout = static_cast<taco::u32x2*>(payload);
            auto* sout = static_cast<taco::f32x2*>(scales);
#define TACO_LAUNCH_COMPRESS(RB, SUB)                                                                           \
            if (two)                                                                                            \
                hipLaunchKernelGGL((taco::compress_mfma_kernel<RB, SUB, 2, true>), dim3(waves), dim3(64), 0, st, \
                                   xin, n_tiles, p->tau, p->eps, pout, sout);                                   \
            else                                                                                                \
                hipLaunchKernelGGL((taco::compress_mfma_kernel<RB, SUB, 1, true>), dim3(waves), dim3(64), 0, st, \
                                   xin, n_tiles, p->tau, p->eps, pout, sout)
            switch (B) {
                case 32: TACO_LAUNCH_COMPRESS(1, 4); break;
                case 64: TACO_LAUNCH_COMPRESS(1, 2); break;
                case 128: TACO_LAUNCH_COMPRESS(1, 1); break;
                case 256: TACO_LAUNCH_COMPRESS(2, 1); break;
                default: TACO_LAUNCH_COMPRESS(4, 1); break;
            }
#undef TACO_LAUNCH_COMPRESS
            if (int rc = launch_status()) return rc;
        }
        first_block = n_tiles * (taco::kTileElems / B);
    }
    const int64_t rest = n_blocks - first_block;
    if (rest > 0) {
        const float tau = p->tau, eps = p->eps;
        int rc = dispatch_block(B, [&](auto bc) {
            constexpr int kB = decltype(bc)::value;
            hipLaunchKernelGGL(taco::compress_butterfly_kernel<kB>, dim3(grid_for(rest, 32)), dim3(64), 0, st,
                               static_cast<const uint16_t*>(x_bf16), n, first_block, rest, tau, eps,
                               static_cast<uint8_t*>(payload), static_cast<float2*>(scales));
        });
        if (rc) return rc;
        if (int rc2 = launch_status()) return rc2;
    }
    return TACO_OK;
}

int taco_decompress_sum(const void* const* payloads, const void* const* scales, int32_t k,
                        int64_t rows, int64_t cols, const taco_params* p, void* out_bf16,
                        void* stream) {
    if (!payloads || !scales || !out_bf16) return TACO_ERR_NULL;
    if (k < 1 || k > TACO_MAX_K) return TACO_ERR_K;
    int64_t n = 0;
    if (int rc = check_common(rows, cols, p, &n)) return rc;
    taco::PayloadTable tab{};
    for (int i = 0; i < k; ++i) {
        if (!payloads[i] || !scales[i]) return TACO_ERR_NULL;
        if (!aligned16(payloads[i]) || !aligned16(scales[i])) return TACO_ERR_ALIGN;
        tab.payload[i] = payloads[i];
        tab.scales[i] = scales[i];
    }
    if (!aligned16(out_bf16)) return TACO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int B = p->block;
    const int64_t n_blocks = (n + B - 1) / B;
    int64_t first_block = 0;
    if (use_mfma(p)) {
        const int64_t n_tiles = n / taco::kTileElems;
        if (n_tiles > 0) {
            // Two output tiles per wave and a ring of four (tile, payload) items in flight: measured
            // best on MI355X for k = 1 and k = 8 (1..16 tiles, rings of 2..8 tried).
            const int tiles_per_wave = 2;
            const unsigned waves = static_cast<unsigned>((n_tiles + tiles_per_wave - 1) / tiles_per_wave);
            auto* o = static_cast<taco::u32x4*>(out_bf16);
#define TACO_LAUNCH_DECODE(RB, SUB)                                                                            \
            hipLaunchKernelGGL((taco::decompress_sum_mfma_kernel<RB, SUB, 4, true, false>), dim3(waves), dim3(64), 0, st, \
                               tab, static_cast<int>(k), n_tiles, tiles_per_wave, o, 0.0f, 0.0f, nullptr, nullptr)
            switch (B) {
                case 32: TACO_LAUNCH_DECODE(1, 4); break;
                case 64: TACO_LAUNCH_DECODE(1, 2); break;
                case 128: TACO_LAUNCH_DECODE(1, 1); break;
                case 256: TACO_LAUNCH_DECODE(2, 1); break;
                default: TACO_LAUNCH_DECODE(4, 1); break;
            }
#undef TACO_LAUNCH_DECODE
            if (int rc = launch_status()) return rc;
        }
        first_block = n_tiles * (taco::kTileElems / B);
    }
    const int64_t rest = n_blocks - first_block;
    if (rest > 0) {
        int rc = dispatch_block(B, [&](auto bc) {
            constexpr int kB = decltype(bc)::value;
            hipLaunchKernelGGL(taco::decompress_sum_butterfly_kernel<kB>, dim3(grid_for(rest, 32)), dim3(64), 0, st,
                               tab, static_cast<int>(k), n, first_block, rest, static_cast<uint16_t*>(out_bf16));
        });
        if (rc) return rc;
        if (int rc2 = launch_status()) return rc2;
    }
    return TACO_OK;
}

int taco_decompress_sum_compress(const void* const* payloads, const void* const* scales, int32_t k,
                                 int64_t rows, int64_t cols, const taco_params* p, void* payload_out,
                                 void* scales_out, void* stream) {
    if (!payloads || !scales || !payload_out || !scales_out) return TACO_ERR_NULL;
    if (k < 1 || k > TACO_MAX_K) return TACO_ERR_K;
    int64_t n = 0;
    if (int rc = check_common(rows, cols, p, &n)) return rc;
    if (!(p->tau > 0.0f) || !(p->eps >= 0.0f) || !std::isfinite(p->tau) || !std::isfinite(p->eps)) return TACO_ERR_PARAM;
    taco::PayloadTable tab{};
    for (int i = 0; i < k; ++i) {
        if (!payloads[i] || !scales[i]) return TACO_ERR_NULL;
        if (!aligned16(payloads[i]) || !aligned16(scales[i])) return TACO_ERR_ALIGN;
        tab.payload[i] = payloads[i];
        tab.scales[i] = scales[i];
    }
    if (!aligned16(payload_out) || !aligned16(scales_out)) return TACO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int B = p->block;
    const int64_t n_blocks = (n + B - 1) / B;
    int64_t first_block = 0;
    if (use_mfma(p)) {
        const int64_t n_tiles = n / taco::kTileElems;
        if (n_tiles > 0) {
            const int tiles_per_wave = 2;
            const unsigned waves = static_cast<unsigned>((n_tiles + tiles_per_wave - 1) / tiles_per_wave);
            auto* pout = static_cast<taco::u32x2*>(payload_out);
            auto* sout = static_cast<taco::f32x2*>(scales_out);
#define TACO_LAUNCH_FUSED(RB, SUB)                                                                             \
            hipLaunchKernelGGL((taco::decompress_sum_mfma_kernel<RB, SUB, 4, true, true>), dim3(waves), dim3(64), 0, st,  \
                               tab, static_cast<int>(k), n_tiles, tiles_per_wave, nullptr, p->tau, p->eps, pout, sout)
            switch (B) {
                case 32: TACO_LAUNCH_FUSED(1, 4); break;
                case 64: TACO_LAUNCH_FUSED(1, 2); break;
                case 128: TACO_LAUNCH_FUSED(1, 1); break;
                case 256: TACO_LAUNCH_FUSED(2, 1); break;
                default: TACO_LAUNCH_FUSED(4, 1); break;
            }
#undef TACO_LAUNCH_FUSED
            if (int rc = launch_status()) return rc;
        }
        first_block = n_tiles * (taco::kTileElems / B);
    }
    const int64_t rest = n_blocks - first_block;
    if (rest > 0) {
        const float tau = p->tau, eps = p->eps;
        int rc = dispatch_block(B, [&](auto bc) {
            constexpr int kB = decltype(bc)::value;
            hipLaunchKernelGGL(taco::decompress_sum_compress_butterfly_kernel<kB>, dim3(grid_for(rest, 32)), dim3(64), 0, st,
                               tab, static_cast<int>(k), n, first_block, rest, tau, eps,
                               static_cast<uint8_t*>(payload_out), static_cast<float2*>(scales_out));
        });
        if (rc) return rc;
        if (int rc2 = launch_status()) return rc2;
    }
    return TACO_OK;
}

int taco_decompress(const void* payload, const void* scales, int64_t rows, int64_t cols,
                    const taco_params* p, void* out_bf16, void* stream) {
    const void* pl[1] = {payload};
    const void* sc[1] = {scales};
    if (!payload || !scales) return TACO_ERR_NULL;
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

const char* taco_strerror(int status) {
    switch (status) {
        case TACO_OK: return "ok";
        case TACO_ERR_NULL: return "null pointer";
        case TACO_ERR_SHAPE: return "bad shape: rows and cols must be positive and rows*cols at most 2^40";
        case TACO_ERR_BLOCK: return "bad block size: must be 32, 64, 128, 256 or 512";
        case TACO_ERR_ALIGN: return "data pointer is not 16-byte aligned";
        case TACO_ERR_K: return "k must be between 1 and 16";
        case TACO_ERR_FORMAT: return "unsupported format: only FP8 E4M3";
        case TACO_ERR_LAUNCH: return "kernel launch failed";
        case TACO_ERR_IMPL: return "requested kernel does not exist for this block size";
        case TACO_ERR_PARAM: return "bad parameter: tau must be positive and eps non-negative, both finite";
        default: return "unknown status";
    }
}

const char* taco_version(void) { return "0.1"; }

}  // extern "C"
