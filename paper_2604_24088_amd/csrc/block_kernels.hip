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

// Calls f(kInterleaved, kFormat, kGeneric) with the three as compile-time constants and returns its result.
// kGeneric = false: the method and its no-rescaling variant (modes 7 and 6), the lean instantiation.
template <typename F>
int with_variant(const Call& call, F&& f) {
    using std::integral_constant;
    auto with_generic = [&](auto layout, auto fmt) {
        return (call.mode & 6) == 6 ? f(layout, fmt, std::false_type{}) : f(layout, fmt, std::true_type{});
    };
    auto with_format = [&](auto layout) {
        if (call.format == 1) return with_generic(layout, integral_constant<int, 1>{});
        if (call.format == 2) return with_generic(layout, integral_constant<int, 2>{});
        return with_generic(layout, integral_constant<int, 0>{});
    };
    return call.interleaved ? with_format(std::true_type{}) : with_format(std::false_type{});
}

int compress(const CompressTable& tab, int count, int64_t workgroups, const Call& call, hipStream_t st) {
    const dim3 grid(static_cast<unsigned>(workgroups)), block(64);
    if (call.mfma) {
        return with_variant(call, [&](auto layout, auto fmt, auto generic) {
            return launch(compress_mfma_kernel<kRB, kSub, decltype(layout)::value, decltype(fmt)::value, decltype(generic)::value>, grid,
                          block, st, tab, count, call.tau, call.eps, call.mode);
        });
    }
    return launch(compress_butterfly_kernel<kB>, grid, block, st, tab, count, call.tau, call.eps, call.interleaved,
                  Variant{call.mode, call.format});
}

int decode(const DecodeTable& tab, int count, int k, int64_t workgroups, const Call& call, bool recompress, bool wide, int tiles_per_wave,
           hipStream_t st) {
    const dim3 grid(static_cast<unsigned>(workgroups));
    if (call.mfma) {
        return with_variant(call, [&](auto layout, auto fmt, auto generic) {
            constexpr bool kIl = decltype(layout)::value, kGen = decltype(generic)::value;
            constexpr int kFmt = decltype(fmt)::value;
            // the fused form of the variants keeps three items in flight instead of four: with four it needs more than
            // 256 registers and only one wave fits a SIMD (measured: 465 us instead of 333 us on the bench tensors)
            if (recompress)
                return launch(decompress_sum_mfma_kernel<kRB, kSub, kGen ? 3 : 4, kIl, true, 1, kFmt, kGen>, grid, dim3(64), st, tab, count, k,
                              tiles_per_wave, call.tau, call.eps, call.mode);
            // Plain decode of the method itself (kGen = false): one payload goes to the kernel with one running sign
            // tile (three (tile, payload) items in flight per wave, three waves per SIMD), more to the kernel with
            // the sign table (four items, two waves per SIMD).  The variants (kGen = true) use the table kernel
            // that also knows how to leave the rotation out.
            if (wide)
                return launch(decompress_sum_mfma_kernel<kRB, kSub, 4, kIl, false, 2, kFmt, kGen>, grid, dim3(128), st, tab, count, k,
                              tiles_per_wave, 0.0f, 0.0f, call.mode);
            if (!kGen && k == 1)
                return launch(decompress_sum_mfma_kernel<kRB, kSub, 3, kIl, false, 1, kFmt, false, true>, grid, dim3(64), st, tab, count, k,
                              tiles_per_wave, 0.0f, 0.0f, call.mode);
            return launch(decompress_sum_mfma_kernel<kRB, kSub, 4, kIl, false, 1, kFmt, kGen>, grid, dim3(64), st, tab, count, k,
                          tiles_per_wave, 0.0f, 0.0f, call.mode);
        });
    }
    const Variant var{call.mode, call.format};
    if (recompress)
        return launch(decompress_sum_compress_butterfly_kernel<kB>, grid, dim3(64), st, tab, count, k, call.tau, call.eps,
                      call.interleaved, var);
    return launch(decompress_sum_butterfly_kernel<kB>, grid, dim3(64), st, tab, count, k, call.interleaved, var);
}

}  // namespace

template <> int launch_compress_b<kB>(const CompressTable& tab, int count, int64_t workgroups, const Call& call, hipStream_t st) {
    return compress(tab, count, workgroups, call, st);
}
template <> int launch_decode_b<kB>(const DecodeTable& tab, int count, int k, int64_t workgroups, const Call& call, bool recompress,
                                    bool wide, int tiles_per_wave, hipStream_t st) {
    return decode(tab, count, k, workgroups, call, recompress, wide, tiles_per_wave, st);
}

}  // namespace taco
