/*
 * taco_debug.h - diagnostic entry points of libtaco_hip (not part of the operator).
 *
 * They exist for tests and benchmarks: the hardware conversion on its own, so that it can be checked
 * against a code table before any kernel is trusted, and two bandwidth yardsticks.  Conventions as in
 * taco.h: device pointers owned by the caller, 16-byte aligned, `stream` a hipStream_t, one kernel
 * per call, status codes of taco_status.
 */
#ifndef TACO_DEBUG_H_
#define TACO_DEBUG_H_

#include "taco.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Diagnostic: converts n device floats to E4M3 codes with the same hardware conversion
 * the compression kernels use (Cvt_FP8 of Eq. quantization), so that it can be compared
 * against a code table.  in_f32: device, n floats; out_codes: device, n bytes; n at most 2^31. */
int taco_debug_cvt_e4m3(const void* in_f32, int64_t n, void* out_codes, void* stream);

/* Diagnostic: plain device-to-device copy of `bytes` bytes (a multiple of 16) with 16-byte
 * loads and stores.  A yardstick for the memory system (reads `bytes`, writes `bytes`) and
 * the known-size kernel that calibrates hardware traffic counters.  src, dst: device. */
int taco_debug_copy(const void* src, void* dst, int64_t bytes, void* stream);

/* Diagnostic: the memory traffic of the operator without its arithmetic, as a yardstick for
 * what the memory system gives a kernel with that mix of reads and writes (Section 4.4.1 puts the
 * cost of the method in its passes over memory).  For each of n_tiles tiles one wave reads
 * src_chunks 16-byte words from each of the k sources (tile t of source i starts at byte
 * t * src_chunks * 16 of srcs[i]) and writes dst_chunks 16-byte words (tile t at byte
 * t * dst_chunks * 16 of dst); the written words are XORs of the loaded ones.  With tiles of 2048
 * elements and block 128: compress is k = 1, src_chunks = 256 (4 KiB of bf16), dst_chunks = 136
 * (2048 codes + 16 pairs of scalars); decompress_sum is k sources of 136 chunks, dst_chunks = 256.
 * srcs: host array of k device pointers, each at least n_tiles * src_chunks * 16 bytes; dst:
 * device, n_tiles * dst_chunks * 16 bytes; 1 <= k <= TACO_MAX_K; 1 <= src_chunks, dst_chunks <= 256.
 * Errors: TACO_ERR_NULL, TACO_ERR_K, TACO_ERR_SHAPE (chunk counts or n_tiles out of range),
 * TACO_ERR_ALIGN, TACO_ERR_LAUNCH. */
int taco_debug_traffic(const void* const* srcs, int32_t k, int32_t src_chunks, void* dst,
                       int32_t dst_chunks, int64_t n_tiles, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TACO_DEBUG_H_ */
