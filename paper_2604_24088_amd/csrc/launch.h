// Launchers of the operator's kernels, one set per block size.  block_kernels.hip defines them (it is
// compiled once per block size with -DTACO_BLOCK=B, so the five sets build in parallel); taco_api.hip
// calls them.  Host-side only.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <tuple>
#include <utility>

#include "tables.h"

namespace taco {

// What a call asks for besides its tensors (taco_params without the block size).
struct Call {
    int format;          // TACO_FORMAT_*
    int mode;            // TACO_MODE_* bit mask
    bool interleaved;    // payload layout
    bool mfma;           // matrix-core kernels (else the butterfly family)
    float tau, eps;
};

// Launches `kernel` and returns 0 or -7 (TACO_ERR_LAUNCH): the status of THIS launch, i.e. the runtime's own
// return value, not the thread's sticky last-error slot (which unrelated earlier work may have set, and which
// is left alone).
template <typename... Params, typename... Args>
int launch(void (*kernel)(Params...), dim3 grid, dim3 block, hipStream_t stream, Args&&... args) {
    static_assert(sizeof...(Params) == sizeof...(Args), "argument count");
    std::tuple<Params...> values{static_cast<Params>(std::forward<Args>(args))...};
    return std::apply(
        [&](auto&... v) {
            void* ptrs[] = {static_cast<void*>(&v)...};
            return hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, ptrs, 0, stream) == hipSuccess ? 0 : -7;
        },
        values);
}

// `workgroups` = size of the grid; the tables say which tensors it covers (tables.h).
template <int B> int launch_compress_b(const CompressTable& tab, int count, int64_t workgroups, const Call& call, hipStream_t st);
// recompress: decompress_sum followed by compress; wide: two waves per workgroup (matrix-core kernels only).
template <int B> int launch_decode_b(const DecodeTable& tab, int count, int k, int64_t workgroups, const Call& call, bool recompress,
                                     bool wide, int tiles_per_wave, hipStream_t st);

}  // namespace taco
