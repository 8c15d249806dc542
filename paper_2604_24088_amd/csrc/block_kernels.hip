// The operator's kernels for ONE block size (TACO_BLOCK = 32, 64, 128, 256 or 512, given on the
// command line) and the launchers that pick the instantiation a call needs.  Compiled once per
// block size; the five objects are independent, so they build in parallel.

#include <hip/hip_runtime.h>

#include <type_traits>

#include "butterfly_kernels.h"
#include "launch.h"
#include "mfma_kernels.h"

#ifndef TACO_BLOCK
#error "compile with -DTACO_BLOCK=32|64|128|256|512"
#endif

namespace taco {
namespace {

constexpr int kB = TACO_BLOCK;
constexpr int kRB = kB > 128 ? kB / 128 : 1;      // units of 128 per block
constexpr int kSub = kB < 128 ? 128 / kB : 1;     // blocks per unit

// Calls f(kInterleaved, kFormat) with the two as compile-time constants and returns its result.
template <typename F>
int with_layout_and_format(const Call& call, F&& f) {
    using std::integral_constant;
    auto with_format = [&](auto layout) {
        if (call.format == 1) return f(layout, integral_constant<int, 1>{});
        if (call.format == 2) return f(layout, integral_constant<int, 2>{});
        return f(layout, integral_constant<int, 0>{});
    };
    return call.interleaved ? with_format(std::true_type{}) : with_format(std::false_type{});
}

template <typename Table>
int compress(const Table& tab, int count, int64_t workgroups, const Call& call, hipStream_t st) {
    const dim3 grid(static_cast<unsigned>(workgroups)), block(64);
    if (call.mfma) {
        const bool rescale = (call.mode & 1) != 0;
        return with_layout_and_format(call, [&](auto layout, auto fmt) {
            return launch(compress_mfma_kernel<kRB, kSub, decltype(layout)::value, decltype(fmt)::value, Table>, grid, block, st, tab,
                          count, call.tau, call.eps, rescale);
        });
    }
    return launch(compress_butterfly_kernel<kB, Table>, grid, block, st, tab, count, call.tau, call.eps, call.interleaved,
                  Variant{call.mode, call.format});
}

template <typename Table>
int decode(const Table& tab, int count, int k, int64_t workgroups, const Call& call, bool recompress, bool wide, int tiles_per_wave,
           hipStream_t st) {
    const dim3 grid(static_cast<unsigned>(workgroups));
    if (call.mfma) {
        const bool rescale = (call.mode & 1) != 0;
        return with_layout_and_format(call, [&](auto layout, auto fmt) {
            constexpr bool kIl = decltype(layout)::value;
            constexpr int kFmt = decltype(fmt)::value;
            if (recompress)
                return launch(decompress_sum_mfma_kernel<kRB, kSub, 4, kIl, true, 1, kFmt, Table>, grid, dim3(64), st, tab, count, k,
                              tiles_per_wave, call.tau, call.eps, rescale);
            if (wide)
                return launch(decompress_sum_mfma_kernel<kRB, kSub, 4, kIl, false, 2, kFmt, Table>, grid, dim3(128), st, tab, count, k,
                              tiles_per_wave, 0.0f, 0.0f, true);
            return launch(decompress_sum_mfma_kernel<kRB, kSub, 4, kIl, false, 1, kFmt, Table>, grid, dim3(64), st, tab, count, k,
                          tiles_per_wave, 0.0f, 0.0f, true);
        });
    }
    const Variant var{call.mode, call.format};
    if (recompress)
        return launch(decompress_sum_compress_butterfly_kernel<kB, Table>, grid, dim3(64), st, tab, count, k, call.tau, call.eps,
                      call.interleaved, var);
    return launch(decompress_sum_butterfly_kernel<kB, Table>, grid, dim3(64), st, tab, count, k, call.interleaved, var);
}

}  // namespace

template <> int launch_compress_b<kB>(const CompressSingle& tab, int count, int64_t workgroups, const Call& call, hipStream_t st) {
    return compress(tab, count, workgroups, call, st);
}
template <> int launch_compress_b<kB>(const CompressBatch& tab, int count, int64_t workgroups, const Call& call, hipStream_t st) {
    return compress(tab, count, workgroups, call, st);
}
template <> int launch_decode_b<kB>(const DecodeSingle& tab, int count, int k, int64_t workgroups, const Call& call, bool recompress,
                                    bool wide, int tiles_per_wave, hipStream_t st) {
    return decode(tab, count, k, workgroups, call, recompress, wide, tiles_per_wave, st);
}
template <> int launch_decode_b<kB>(const DecodeBatch& tab, int count, int k, int64_t workgroups, const Call& call, bool recompress,
                                    bool wide, int tiles_per_wave, hipStream_t st) {
    return decode(tab, count, k, workgroups, call, recompress, wide, tiles_per_wave, st);
}

}  // namespace taco
