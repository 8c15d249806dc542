/*
 * taco.h - C ABI of the MI355X (gfx950) implementation of the TACO fused FP8
 * compression operator for tensor-parallel intermediate tensors.
 *
 * The operator is the one the TACO paper defines in Section 4:
 *   - the flattened bf16 tensor is cut into contiguous blocks of B elements
 *     (Section 4.2.2, Eq. ash_partition);
 *   - each block is rescaled by alpha_k = tau / sigma_k, sigma_k its RMS with eps inside
 *     the root (Eq. ash_sigma, Eq. ash_alpha), and rotated by the orthonormal Hadamard
 *     matrix (Eq. ash_rotation): together the Adaptive Scale-Hadamard transform;
 *   - Dual-Scale quantisation (Section 4.3): s_k = max|Z_k| / Q_max (Eq. post_scale),
 *     codes = Cvt_FP8(Z_k / s_k) (Eq. quantization);
 *   - the receiver undoes the three steps in reverse order (Eqs. recon_dequant,
 *     recon_ifwht, recon_rescale), in one fused kernel (Section 4.4.1);
 *   - k decoded payloads are added in one local reduction (Section 4.4.2, the
 *     ReduceScatter half of the two-shot AllReduce).
 * Algorithm 1 of the paper lists the sender and receiver sides step by step.
 *
 * Conventions for every entry point
 *   - All data pointers are DEVICE pointers owned by the caller; the library allocates
 *     nothing, keeps no state and never synchronises.  `stream` is a hipStream_t (NULL =
 *     the default stream); each call enqueues its kernels on it and returns.
 *   - Inputs and outputs must not overlap.  Data pointers must be 16-byte aligned.
 *   - A tensor of `rows` x `cols` bf16 values is row-major and is treated as the flat
 *     vector of n = rows*cols elements; blocks may straddle rows.  When n is not a
 *     multiple of B the last block is zero padded (sigma still divides by B).
 *   - FP8 is (unless params->format says otherwise) E4M3 in the OCP 8-bit layout (1 sign, 4 exponent bits with bias 7, 3
 *     mantissa bits, subnormals, no infinities, Q_max = 448), round to nearest even.
 *   - Hadamard matrix: natural (Sylvester) order, H[i][j] = (-1)^popcount(i & j).
 *   - Payload layout: ceil(n/B)*B one-byte codes, code i of block k at byte k*B + i.
 *     Scales layout: ceil(n/B) records { float alpha_k; float s_k; }.
 *     The two regions may be adjacent parts of one allocation (the paper's contiguous
 *     metadata placement, Section 4.4.2, in structure-of-arrays form).
 *   - A block whose rotated maximum is zero stores s_k = 0 and zero codes (sign bits
 *     of the codes are unspecified) and decodes to zeros.
 *   - Non-finite inputs are outside the contract, and so are blocks whose sum of squares
 *     leaves the range of normal fp32 numbers (|x| up to about 2^60 and down to 2^-60 are
 *     tested): the kernels work in fp32.
 *   - Return value: TACO_OK (0) or a negative taco_status.  Argument errors are found on
 *     the host before anything is launched.
 */
#ifndef TACO_H_
#define TACO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TACO_MAX_K 16 /* most payloads one taco_decompress_sum call can add */

typedef enum taco_status {
    TACO_OK = 0,
    TACO_ERR_NULL = -1,   /* a required pointer is NULL                               */
    TACO_ERR_SHAPE = -2,  /* rows <= 0, cols <= 0 or rows*cols overflows 2^40        */
    TACO_ERR_BLOCK = -3,  /* block is not one of 32, 64, 128, 256, 512                */
    TACO_ERR_ALIGN = -4,  /* a data pointer is not 16-byte aligned                    */
    TACO_ERR_K = -5,      /* k outside 1..TACO_MAX_K                                  */
    TACO_ERR_FORMAT = -6, /* params->format is not one of TACO_FORMAT_*               */
    TACO_ERR_LAUNCH = -7, /* the HIP runtime refused the launch (hipGetLastError)     */
    TACO_ERR_IMPL = -8,   /* params->impl is not one of TACO_IMPL_*, or MFMA was forced
                             for an ablation variant                                  */
    TACO_ERR_PARAM = -9,  /* tau <= 0, eps < 0, or a non-finite parameter             */
    TACO_ERR_LAYOUT = -10,/* params->layout is not one of TACO_LAYOUT_*               */
    TACO_ERR_MODE = -11   /* params->mode is outside 0..TACO_MODE_FULL                */
} taco_status;

/* Code book.  E4M3 is the method's (chosen by the paper's format ablation, Section 5.3); E5M2
 * (OCP: bias 15, Q_max 57344) and INT8 (round(x / Delta), Delta = max|x| / 127, Section 2.3) are the
 * two alternatives that ablation compares against. */
enum { TACO_FORMAT_E4M3 = 0, TACO_FORMAT_E5M2 = 1, TACO_FORMAT_INT8 = 2 };

/* Stages of the method, for the paper's component ablations (Section 5.2.2, Section 5.3): a bit
 * mask.  Without RESCALE alpha_k = 1; without ROTATE Z_k = alpha_k G_k; without POSTSCALE s_k = 1
 * and Z_k itself is converted, saturating at +-Q_max.  FULL (7) is the method; 0 is the direct
 * cast, 4 dual scale only, 2 the standard Hadamard transform, 3 ASH without DS.  The matrix-core
 * kernels cover the variants that keep the method's structure (rotation and post-rotation scale
 * on, i.e. modes 7 and 6, in E4M3 or E5M2); every other variant runs on the butterfly kernels. */
enum { TACO_MODE_RESCALE = 1, TACO_MODE_ROTATE = 2, TACO_MODE_POSTSCALE = 4, TACO_MODE_FULL = 7 };

/* Kernel selection.  AUTO runs whole tiles of 2048 elements on the matrix-core kernels where the
 * variant allows it (see above) and the rest of the tensor on the butterfly kernels; MFMA is AUTO
 * that fails with TACO_ERR_IMPL for a variant the matrix-core kernels do not cover; BUTTERFLY runs
 * everything on the butterfly kernels (kept for tests and benchmarks that compare the two). */
enum { TACO_IMPL_AUTO = 0, TACO_IMPL_BUTTERFLY = 1, TACO_IMPL_MFMA = 2 };

/* Where the two scalars of a block travel (Section 4.4.2 of the paper places them directly
 * behind the block's codes).
 *   SPLIT        `payload` = the codes of all blocks in element order, `scales` = the records
 *                {alpha, s} of all blocks.  The two regions may be adjacent parts of one buffer.
 *   INTERLEAVED  `payload` = one record of B + 8 bytes per block: B codes, float alpha, float s.
 *                Its size is taco_payload_bytes + taco_scales_bytes; every `scales` argument is
 *                ignored and may be NULL.  Records are 8-byte but not 16-byte aligned. */
enum { TACO_LAYOUT_SPLIT = 0, TACO_LAYOUT_INTERLEAVED = 1 };

/* Hyper-parameters of Algorithm 1 (its input line): block size B, target energy tau,
 * stabiliser eps; Q_max follows from the format. */
typedef struct taco_params {
    int32_t block;  /* B: 32, 64, 128, 256 or 512                                  */
    float tau;      /* tau of Eq. ash_alpha, > 0 (the paper gives no value; 1.0f)  */
    float eps;      /* eps of Eq. ash_sigma, >= 0 (the paper gives no value; 1e-12f).  With eps = 0 an
                       all-zero block stores alpha = inf, s = 0 and still decodes to zeros */
    int32_t format; /* TACO_FORMAT_*                                               */
    int32_t impl;   /* TACO_IMPL_*                                                 */
    int32_t layout; /* TACO_LAYOUT_*                                               */
    int32_t mode;   /* TACO_MODE_* bit mask, TACO_MODE_FULL for the method         */
} taco_params;

/* Fills *p with B = 128, tau = 1, eps = 1e-12, E4M3, AUTO, SPLIT, FULL. */
void taco_default_params(taco_params* p);

/* Sizes of the two output regions of taco_compress for n elements: ceil(n/B)*B bytes of
 * codes and ceil(n/B)*8 bytes of {alpha, s} records.  0 if n <= 0 or block is invalid. */
size_t taco_payload_bytes(int64_t n, int32_t block);
size_t taco_scales_bytes(int64_t n, int32_t block);

/* Sender side of Algorithm 1 (fused compression kernel, Section 4.4.1).
 *   x_bf16   in   device, rows*cols bf16 values
 *   payload  out  device, taco_payload_bytes(rows*cols, B) bytes
 *   scales   out  device, taco_scales_bytes(rows*cols, B) bytes
 * Errors, all found before anything is launched except the last: TACO_ERR_NULL, _SHAPE, _BLOCK,
 * _FORMAT, _MODE, _IMPL, _LAYOUT, _PARAM (tau, eps), _ALIGN; TACO_ERR_LAUNCH from the runtime. */
int taco_compress(const void* x_bf16, int64_t rows, int64_t cols, const taco_params* p,
                  void* payload, void* scales, void* stream);

/* Receiver side of Algorithm 1 (fused decompression kernel, Section 4.1 / 4.4.1):
 * out = bf16( H (codes * s) / sqrt(B) / alpha ).  tau and eps are ignored.
 *   out_bf16 out  device, rows*cols bf16 values
 * Errors: as taco_compress without TACO_ERR_PARAM. */
int taco_decompress(const void* payload, const void* scales, int64_t rows, int64_t cols,
                    const taco_params* p, void* out_bf16, void* stream);

/* Receiver side followed by the single local reduction of Section 4.4.2:
 * out = bf16( sum_{i<k} decode(payloads[i], scales[i]) ), accumulated in fp32 with one
 * final rounding.  `payloads` and `scales` are HOST arrays of k device pointers, read
 * during the call (they may be freed as soon as it returns).  k = 1 equals taco_decompress.
 * Errors: as taco_decompress, and TACO_ERR_K for k outside 1..TACO_MAX_K; a NULL or misaligned
 * entry of the arrays is TACO_ERR_NULL / TACO_ERR_ALIGN. */
int taco_decompress_sum(const void* const* payloads, const void* const* scales, int32_t k,
                        int64_t rows, int64_t cols, const taco_params* p, void* out_bf16,
                        void* stream);

/* Receive side of the reduce-scatter immediately followed by the send side of the all-gather
 * (Section 4.4.2: the two-shot AllReduce is ReduceScatter + AllGather, and the reduced shard is
 * compressed again for the AllGather).  Equals taco_decompress_sum into a bf16 tensor followed by
 * taco_compress of that tensor, bit for bit, but the bf16 tensor never reaches device memory.
 *   payloads, scales  in   HOST arrays of k device pointers (as for taco_decompress_sum)
 *   payload_out       out  device, taco_payload_bytes(rows*cols, B) bytes
 *   scales_out        out  device, taco_scales_bytes(rows*cols, B) bytes
 * Outputs must not overlap any input.
 * Errors: as taco_decompress_sum, and TACO_ERR_PARAM (tau and eps are used by the compress half). */
int taco_decompress_sum_compress(const void* const* payloads, const void* const* scales, int32_t k,
                                 int64_t rows, int64_t cols, const taco_params* p, void* payload_out,
                                 void* scales_out, void* stream);

/* Diagnostic: converts n device floats to E4M3 codes with the same hardware conversion
 * the compression kernels use (Cvt_FP8 of Eq. quantization), so that it can be compared
 * against a code table.  in_f32: device, n floats; out_codes: device, n bytes. */
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

/* Text for a taco_status value (static storage, never NULL). */
const char* taco_strerror(int status);

/* Library version, "major.minor". */
const char* taco_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TACO_H_ */
