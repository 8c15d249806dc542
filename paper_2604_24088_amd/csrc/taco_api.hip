// Host side of the C ABI declared in include/taco.h and include/taco_debug.h: argument checks,
// kernel choice, launch geometry.  No device memory is allocated and nothing is synchronised here;
// every entry point enqueues exactly one kernel.  The operator's kernels are instantiated per block
// size in block_kernels.hip (compiled once per block size, in parallel); this file reaches them
// through the launchers declared in launch.h.

#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdint>
#include <type_traits>
#include <utility>

#include "../../include/taco.h"
#include "../../include/taco_debug.h"
#include "debug_kernels.h"
#include "device_util.h"
#include "launch.h"
#include "tables.h"

#ifndef TACO_BUILD_ID
#define TACO_BUILD_ID "unknown"
#endif

static_assert(TACO_MAX_K == taco::kMaxK && TACO_MAX_BATCH == taco::kMaxBatch &&
              TACO_MAX_BATCH_PAYLOADS == taco::kMaxBatchSources, "header and kernel tables disagree");

namespace {

// One launch covers a tensor with one workgroup of 64 or 128 threads per 2048 elements or two tiles; 2^36
// elements keep the thread count of a launch below 2^32.
constexpr int64_t kMaxElems = int64_t(1) << 36;
constexpr int64_t kMaxCvtElems = int64_t(1) << 31;
constexpr int64_t kTileElems = 2048;      // elements per workgroup of the operator's kernels

bool block_ok(int32_t b) { return b == 32 || b == 64 || b == 128 || b == 256 || b == 512; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// The matrix-core kernels implement the method and every ablation variant (any mode, any code book);
// the butterfly kernels, a second and independent family, run only when asked for.

int check_params(const taco_params* p) {
    if (!p) return TACO_ERR_NULL;
    if (!block_ok(p->block)) return TACO_ERR_BLOCK;
    if (p->format != TACO_FORMAT_E4M3 && p->format != TACO_FORMAT_E5M2 && p->format != TACO_FORMAT_INT8) return TACO_ERR_FORMAT;
    if (p->mode < 0 || p->mode > TACO_MODE_FULL) return TACO_ERR_MODE;
    if (p->impl != TACO_IMPL_AUTO && p->impl != TACO_IMPL_BUTTERFLY && p->impl != TACO_IMPL_MFMA) return TACO_ERR_IMPL;
    if (p->layout != TACO_LAYOUT_SPLIT && p->layout != TACO_LAYOUT_INTERLEAVED) return TACO_ERR_LAYOUT;
    return TACO_OK;
}

int check_shape(int64_t rows, int64_t cols, int64_t* n_out) {
    if (rows <= 0 || cols <= 0) return TACO_ERR_SHAPE;
    if (rows > kMaxElems || cols > kMaxElems || rows > kMaxElems / cols) return TACO_ERR_SHAPE;
    *n_out = rows * cols;
    return TACO_OK;
}

bool params_ok_for_compress(const taco_params* p) {
    return p->tau > 0.0f && p->eps >= 0.0f && std::isfinite(p->tau) && std::isfinite(p->eps);
}

bool use_mfma(const taco_params* p) { return p->impl != TACO_IMPL_BUTTERFLY; }

taco::Call call_of(const taco_params* p) {
    return taco::Call{p->format, p->mode, p->layout == TACO_LAYOUT_INTERLEAVED, use_mfma(p), p->tau, p->eps};
}

// ---- byte ranges, for the overlap test ------------------------------------------------------------

struct Range {
    uintptr_t lo, hi;      // [lo, hi)
};

Range range_of(const void* p, uint64_t bytes) {
    const uintptr_t a = reinterpret_cast<uintptr_t>(p);
    return Range{a, a + bytes};
}

bool overlap(const Range& a, const Range& b) { return a.lo < b.hi && b.lo < a.hi; }

uint64_t blocks_of(int64_t n, int B) { return static_cast<uint64_t>((n + B - 1) / B); }
// Bytes of the payload argument (codes, or records in the interleaved layout) and of the scales argument.
uint64_t payload_arg_bytes(int64_t n, const taco_params* p) {
    return blocks_of(n, p->block) * static_cast<uint64_t>(p->layout == TACO_LAYOUT_INTERLEAVED ? p->block + 8 : p->block);
}
uint64_t scales_arg_bytes(int64_t n, const taco_params* p) {
    return p->layout == TACO_LAYOUT_INTERLEAVED ? 0 : blocks_of(n, p->block) * 8u;
}

// Up to kMaxRanges ranges of each kind per call; an output may overlap neither an input nor another output.
struct RangeSet {
    static constexpr int kMaxRanges = 2 * TACO_MAX_BATCH_PAYLOADS + 2 * TACO_MAX_BATCH;
    Range in[kMaxRanges];
    Range out[kMaxRanges];
    int n_in = 0, n_out = 0;
    void add_in(const void* p, uint64_t bytes) { if (p && bytes && n_in < kMaxRanges) in[n_in++] = range_of(p, bytes); }
    void add_out(const void* p, uint64_t bytes) { if (p && bytes && n_out < kMaxRanges) out[n_out++] = range_of(p, bytes); }
    bool clash() const {
        for (int o = 0; o < n_out; ++o) {
            for (int i = 0; i < n_in; ++i)
                if (overlap(out[o], in[i])) return true;
            for (int q = o + 1; q < n_out; ++q)
                if (overlap(out[o], out[q])) return true;
        }
        return false;
    }
};

int64_t tiles_of(int64_t n) { return (n + kTileElems - 1) / kTileElems; }

// ---- compress -----------------------------------------------------------------------------------

// One workgroup (one wave) per tile of 2048 elements in either family: measured best on MI355X at every
// block size and in both layouts (2 tiles per wave cost 4-5 % on the largest tensors, 4 more).
int launch_compress(const taco::CompressTable& tab, int count, int64_t workgroups, const taco_params* p, hipStream_t st) {
    const taco::Call call = call_of(p);
    switch (p->block) {
        case 32: return taco::launch_compress_b<32>(tab, count, workgroups, call, st);
        case 64: return taco::launch_compress_b<64>(tab, count, workgroups, call, st);
        case 128: return taco::launch_compress_b<128>(tab, count, workgroups, call, st);
        case 256: return taco::launch_compress_b<256>(tab, count, workgroups, call, st);
        case 512: return taco::launch_compress_b<512>(tab, count, workgroups, call, st);
        default: return TACO_ERR_BLOCK;
    }
}

int check_compress_item(const void* x, int64_t rows, int64_t cols, void* payload, void* scales, const taco_params* p,
                        int64_t* n, RangeSet* ranges) {
    if (!x || !payload) return TACO_ERR_NULL;
    if (int rc = check_shape(rows, cols, n)) return rc;
    const bool il = p->layout == TACO_LAYOUT_INTERLEAVED;
    if (!il && !scales) return TACO_ERR_NULL;
    if (!aligned16(x) || !aligned16(payload) || (!il && !aligned16(scales))) return TACO_ERR_ALIGN;
    ranges->add_in(x, 2u * static_cast<uint64_t>(*n));
    ranges->add_out(payload, payload_arg_bytes(*n, p));
    if (!il) ranges->add_out(scales, scales_arg_bytes(*n, p));
    return TACO_OK;
}

// ---- decode -------------------------------------------------------------------------------------

struct DecodeShape {
    bool wide;              // two waves per workgroup
    int tiles_per_wave;
    int64_t tiles_per_group;
};

// Launch shape of the matrix-core decode kernels, from measurements on MI355X (bf16 [16384, 12288], every k):
//   plain decode   k = 1: one tile per single-wave workgroup up to block 128 (1 % faster), two tiles above (1-3 %
//                  faster); k = 2 .. 5: two tiles; k >= 6: two waves per workgroup,
//                  one tile each (3-10 % faster than two tiles per wave at k = 8 .. 16, 5-10 % slower at k <= 4);
//   fused form     few payloads leave a wave little work per tile to hide the compress stage behind, so it takes
//                  more tiles: 8 for k <= 3, 3 for k = 4 and 5, 2 from k = 6 on (block 32: 1 from k = 6 on).
//                  More tiles per wave always lower the time of a cache-fed run and, beyond these values, raise the
//                  HBM-fed one: the tiles in flight stop forming one dense window that advances through DRAM.
DecodeShape decode_shape(const taco_params* p, int k, bool recompress) {
    if (!use_mfma(p)) return DecodeShape{false, 1, 1};      // butterfly family: one tile per single-wave workgroup
    if (recompress) {
        const int tiles = k <= 3 ? 8 : k <= 5 ? 3 : p->block == 32 ? 1 : 2;
        return DecodeShape{false, tiles, tiles};
    }
    if (k >= 6) return DecodeShape{true, 1, 2};
    const int tiles = (k == 1 && p->block <= 128) ? 1 : 2;
    return DecodeShape{false, tiles, tiles};
}

int64_t decode_groups(int64_t n, const DecodeShape& shape) {
    return (tiles_of(n) + shape.tiles_per_group - 1) / shape.tiles_per_group;
}

int launch_decode(const taco::DecodeTable& tab, int count, int k, int64_t workgroups, const taco_params* p, bool recompress, hipStream_t st) {
    const taco::Call call = call_of(p);
    const DecodeShape shape = decode_shape(p, k, recompress);
    switch (p->block) {
        case 32: return taco::launch_decode_b<32>(tab, count, k, workgroups, call, recompress, shape.wide, shape.tiles_per_wave, st);
        case 64: return taco::launch_decode_b<64>(tab, count, k, workgroups, call, recompress, shape.wide, shape.tiles_per_wave, st);
        case 128: return taco::launch_decode_b<128>(tab, count, k, workgroups, call, recompress, shape.wide, shape.tiles_per_wave, st);
        case 256: return taco::launch_decode_b<256>(tab, count, k, workgroups, call, recompress, shape.wide, shape.tiles_per_wave, st);
        case 512: return taco::launch_decode_b<512>(tab, count, k, workgroups, call, recompress, shape.wide, shape.tiles_per_wave, st);
        default: return TACO_ERR_BLOCK;
    }
}

// Checks the k sources of one tensor and records their byte ranges.  In the interleaved layout the scales
// live inside the payload and `scales` (the array or its entries) may be NULL.
template <typename Put>
int check_sources(const void* const* payloads, const void* const* scales, int k, int64_t n, const taco_params* p,
                  RangeSet* ranges, Put&& put) {
    const bool il = p->layout == TACO_LAYOUT_INTERLEAVED;
    if (!payloads || (!il && !scales)) return TACO_ERR_NULL;
    for (int i = 0; i < k; ++i) {
        if (!payloads[i] || (!il && !scales[i])) return TACO_ERR_NULL;
        if (!aligned16(payloads[i]) || (!il && !aligned16(scales[i]))) return TACO_ERR_ALIGN;
        ranges->add_in(payloads[i], payload_arg_bytes(n, p));
        if (!il) ranges->add_in(scales[i], scales_arg_bytes(n, p));
        put(i, payloads[i], il ? nullptr : scales[i]);
    }
    return TACO_OK;
}

int decode_single(const void* const* payloads, const void* const* scales, int32_t k, int64_t rows, int64_t cols,
                  const taco_params* p, bool recompress, void* out_bf16, void* payload_out, void* scales_out, void* stream) {
    if (k < 1 || k > TACO_MAX_K) return TACO_ERR_K;
    if (int rc = check_params(p)) return rc;
    int64_t n = 0;
    if (int rc = check_shape(rows, cols, &n)) return rc;
    const bool il = p->layout == TACO_LAYOUT_INTERLEAVED;
    if (recompress) {
        if (!payload_out || (!il && !scales_out)) return TACO_ERR_NULL;
        if (!params_ok_for_compress(p)) return TACO_ERR_PARAM;
    } else if (!out_bf16) {
        return TACO_ERR_NULL;
    }
    RangeSet ranges;
    taco::DecodeTable tab{};
    if (int rc = check_sources(payloads, scales, k, n, p, &ranges, [&](int i, const void* pl, const void* sc) {
            tab.src_payload[i] = pl;
            tab.src_scales[i] = sc;
        }))
        return rc;
    if (recompress) {
        if (!aligned16(payload_out) || (!il && !aligned16(scales_out))) return TACO_ERR_ALIGN;
        ranges.add_out(payload_out, payload_arg_bytes(n, p));
        if (!il) ranges.add_out(scales_out, scales_arg_bytes(n, p));
    } else {
        if (!aligned16(out_bf16)) return TACO_ERR_ALIGN;
        ranges.add_out(out_bf16, 2u * static_cast<uint64_t>(n));
    }
    if (ranges.clash()) return TACO_ERR_OVERLAP;
    tab.out[0] = out_bf16;
    tab.payload_out[0] = payload_out;
    tab.scales_out[0] = il ? nullptr : scales_out;
    tab.n_elems[0] = n;
    const int64_t workgroups = decode_groups(n, decode_shape(p, k, recompress));
    tab.first[1] = workgroups;
    return launch_decode(tab, 1, k, workgroups, p, recompress, static_cast<hipStream_t>(stream));
}

// One tensor of a batched decode: its k sources and either the bf16 output or the re-compressed outputs.
struct BatchItem {
    const void* const* payloads;
    const void* const* scales;
    int64_t rows, cols;
    void* out_bf16;
    void* payload_out;
    void* scales_out;
};

template <typename Get>
int decode_batch(int32_t count, int32_t k, const taco_params* p, bool recompress, void* stream, Get&& get) {
    if (k < 1 || k > TACO_MAX_K) return TACO_ERR_K;
    if (count < 1 || count > TACO_MAX_BATCH || static_cast<int64_t>(count) * k > TACO_MAX_BATCH_PAYLOADS) return TACO_ERR_BATCH;
    if (int rc = check_params(p)) return rc;
    if (recompress && !params_ok_for_compress(p)) return TACO_ERR_PARAM;
    const bool il = p->layout == TACO_LAYOUT_INTERLEAVED;
    const DecodeShape shape = decode_shape(p, k, recompress);
    RangeSet ranges;
    taco::DecodeTable tab{};
    int64_t workgroups = 0;
    for (int t = 0; t < count; ++t) {
        const BatchItem item = get(t);
        int64_t n = 0;
        if (recompress ? (!item.payload_out || (!il && !item.scales_out)) : !item.out_bf16) return TACO_ERR_NULL;
        if (int rc = check_shape(item.rows, item.cols, &n)) return rc;
        if (int rc = check_sources(item.payloads, item.scales, k, n, p, &ranges, [&](int i, const void* pl, const void* sc) {
                tab.src_payload[t * k + i] = pl;
                tab.src_scales[t * k + i] = sc;
            }))
            return rc;
        if (recompress) {
            if (!aligned16(item.payload_out) || (!il && !aligned16(item.scales_out))) return TACO_ERR_ALIGN;
            ranges.add_out(item.payload_out, payload_arg_bytes(n, p));
            if (!il) ranges.add_out(item.scales_out, scales_arg_bytes(n, p));
            tab.payload_out[t] = item.payload_out;
            tab.scales_out[t] = il ? nullptr : item.scales_out;
        } else {
            if (!aligned16(item.out_bf16)) return TACO_ERR_ALIGN;
            ranges.add_out(item.out_bf16, 2u * static_cast<uint64_t>(n));
            tab.out[t] = item.out_bf16;
        }
        tab.n_elems[t] = n;
        tab.first[t] = workgroups;
        workgroups += decode_groups(n, shape);
    }
    tab.first[count] = workgroups;
    if (ranges.clash()) return TACO_ERR_OVERLAP;
    return launch_decode(tab, count, k, workgroups, p, recompress, static_cast<hipStream_t>(stream));
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
    if (int rc = check_params(p)) return rc;
    int64_t n = 0;
    RangeSet ranges;
    if (int rc = check_compress_item(x_bf16, rows, cols, payload, scales, p, &n, &ranges)) return rc;
    if (!params_ok_for_compress(p)) return TACO_ERR_PARAM;
    if (ranges.clash()) return TACO_ERR_OVERLAP;
    const bool il = p->layout == TACO_LAYOUT_INTERLEAVED;
    taco::CompressTable tab{};
    tab.item[0] = taco::CompressItem{x_bf16, payload, il ? nullptr : scales, n};
    tab.first[1] = tiles_of(n);
    return launch_compress(tab, 1, tiles_of(n), p, static_cast<hipStream_t>(stream));
}

int taco_compress_batch(const taco_compress_item* items, int32_t count, const taco_params* p, void* stream) {
    if (!items) return TACO_ERR_NULL;
    if (count < 1 || count > TACO_MAX_BATCH) return TACO_ERR_BATCH;
    if (int rc = check_params(p)) return rc;
    if (!params_ok_for_compress(p)) return TACO_ERR_PARAM;
    const bool il = p->layout == TACO_LAYOUT_INTERLEAVED;
    RangeSet ranges;
    taco::CompressTable tab{};
    int64_t workgroups = 0;
    for (int i = 0; i < count; ++i) {
        int64_t n = 0;
        if (int rc = check_compress_item(items[i].x_bf16, items[i].rows, items[i].cols, items[i].payload, items[i].scales, p, &n,
                                         &ranges))
            return rc;
        tab.item[i] = taco::CompressItem{items[i].x_bf16, items[i].payload, il ? nullptr : items[i].scales, n};
        tab.first[i] = workgroups;
        workgroups += tiles_of(n);
    }
    tab.first[count] = workgroups;
    if (ranges.clash()) return TACO_ERR_OVERLAP;
    return launch_compress(tab, count, workgroups, p, static_cast<hipStream_t>(stream));
}

int taco_decompress_sum(const void* const* payloads, const void* const* scales, int32_t k,
                        int64_t rows, int64_t cols, const taco_params* p, void* out_bf16,
                        void* stream) {
    return decode_single(payloads, scales, k, rows, cols, p, false, out_bf16, nullptr, nullptr, stream);
}

int taco_decompress_sum_compress(const void* const* payloads, const void* const* scales, int32_t k,
                                 int64_t rows, int64_t cols, const taco_params* p, void* payload_out,
                                 void* scales_out, void* stream) {
    return decode_single(payloads, scales, k, rows, cols, p, true, nullptr, payload_out, scales_out, stream);
}

int taco_decompress(const void* payload, const void* scales, int64_t rows, int64_t cols,
                    const taco_params* p, void* out_bf16, void* stream) {
    const void* pl[1] = {payload};
    const void* sc[1] = {scales};
    return decode_single(pl, sc, 1, rows, cols, p, false, out_bf16, nullptr, nullptr, stream);
}

int taco_decompress_sum_batch(const taco_decode_item* items, int32_t count, int32_t k, const taco_params* p,
                              void* stream) {
    if (!items) return TACO_ERR_NULL;
    return decode_batch(count, k, p, false, stream, [&](int t) {
        return BatchItem{items[t].payloads, items[t].scales, items[t].rows, items[t].cols, items[t].out_bf16, nullptr, nullptr};
    });
}

int taco_decompress_sum_compress_batch(const taco_recompress_item* items, int32_t count, int32_t k, const taco_params* p,
                                       void* stream) {
    if (!items) return TACO_ERR_NULL;
    return decode_batch(count, k, p, true, stream, [&](int t) {
        return BatchItem{items[t].payloads, items[t].scales, items[t].rows, items[t].cols, nullptr, items[t].payload_out,
                         items[t].scales_out};
    });
}

int taco_debug_cvt_e4m3(const void* in_f32, int64_t n, void* out_codes, void* stream) {
    if (!in_f32 || !out_codes) return TACO_ERR_NULL;
    if (n <= 0 || n > kMaxCvtElems) return TACO_ERR_SHAPE;
    const int threads = 256;
    const int64_t blocks = (n + threads - 1) / threads;
    return taco::launch(taco::cvt_e4m3_kernel, dim3(static_cast<unsigned>(blocks)), dim3(threads), static_cast<hipStream_t>(stream),
                  static_cast<const float*>(in_f32), n, static_cast<uint8_t*>(out_codes));
}

int taco_debug_copy(const void* src, void* dst, int64_t bytes, void* stream) {
    if (!src || !dst) return TACO_ERR_NULL;
    if (bytes <= 0 || (bytes & 15) != 0) return TACO_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(dst)) return TACO_ERR_ALIGN;
    const int64_t n16 = bytes / 16;
    const int64_t want = (n16 + 255) / 256;
    const int64_t cap = 256 * 32;       // grid-stride copy: 32 workgroups per compute unit of an MI355X
    return taco::launch(taco::copy_kernel, dim3(static_cast<unsigned>(want < cap ? want : cap)), dim3(256), static_cast<hipStream_t>(stream),
                  static_cast<const taco::u32x4*>(src), static_cast<taco::u32x4*>(dst), n16);
}

int taco_debug_traffic(const void* const* srcs, int32_t k, int32_t src_chunks, void* dst,
                       int32_t dst_chunks, int64_t n_tiles, void* stream) {
    if (!srcs || !dst) return TACO_ERR_NULL;
    if (k < 1 || k > TACO_MAX_K) return TACO_ERR_K;
    if (src_chunks < 1 || src_chunks > 256 || dst_chunks < 1 || dst_chunks > 256) return TACO_ERR_SHAPE;
    if (n_tiles < 1 || n_tiles > kMaxElems / kTileElems) return TACO_ERR_SHAPE;
    taco::SourceTable tab{};
    for (int i = 0; i < k; ++i) {
        if (!srcs[i]) return TACO_ERR_NULL;
        if (!aligned16(srcs[i])) return TACO_ERR_ALIGN;
        tab.src[i] = srcs[i];
    }
    if (!aligned16(dst)) return TACO_ERR_ALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    // The launch shapes of the kernels it stands in for: two waves per workgroup from six sources on.
    if (k >= 6)
        return taco::launch(taco::traffic_kernel<2>, dim3(static_cast<unsigned>((n_tiles + 1) / 2)), dim3(128), st, tab, k, src_chunks,
                      static_cast<taco::u32x4*>(dst), dst_chunks, n_tiles);
    return taco::launch(taco::traffic_kernel<1>, dim3(static_cast<unsigned>(n_tiles)), dim3(64), st, tab, k, src_chunks,
                  static_cast<taco::u32x4*>(dst), dst_chunks, n_tiles);
}

const char* taco_strerror(int status) {
    switch (status) {
        case TACO_OK: return "ok";
        case TACO_ERR_NULL: return "null pointer";
        case TACO_ERR_SHAPE: return "bad shape: rows and cols must be positive and rows*cols at most 2^36";
        case TACO_ERR_BLOCK: return "bad block size: must be 32, 64, 128, 256 or 512";
        case TACO_ERR_ALIGN: return "data pointer is not 16-byte aligned";
        case TACO_ERR_K: return "k must be between 1 and 16";
        case TACO_ERR_FORMAT: return "bad format: must be E4M3, E5M2 or INT8";
        case TACO_ERR_LAUNCH: return "kernel launch failed";
        case TACO_ERR_IMPL: return "bad kernel selection: must be AUTO, BUTTERFLY or MFMA";
        case TACO_ERR_PARAM: return "bad parameter: tau must be positive and eps non-negative, both finite";
        case TACO_ERR_LAYOUT: return "bad layout: must be split or interleaved";
        case TACO_ERR_MODE: return "bad mode: must be a combination of the three TACO_MODE_* bits";
        case TACO_ERR_OVERLAP: return "an output buffer overlaps an input or another output";
        case TACO_ERR_BATCH: return "bad batch: 1 to 32 tensors, and at most 128 payloads in all";
        default: return "unknown status";
    }
}

const char* taco_version(void) { return "0.5"; }

const char* taco_build_id(void) {
    // the marker in front lets a build script find the digest in the binary without loading it
    static const char marked[] = "taco-build-id:" TACO_BUILD_ID;
    return marked + sizeof("taco-build-id:") - 1;
}

}  // extern "C"
