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
 *     the default stream); each call enqueues exactly ONE kernel on it and returns.
 *   - Outputs must not overlap inputs or each other: the byte ranges are compared on the host
 *     and an overlap is TACO_ERR_OVERLAP before anything is launched (inputs may overlap or
 *     repeat one another).  Data pointers must be 16-byte aligned.
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
 *   - Range (the kernels work in fp32).  Non-finite inputs are outside the contract.  Where a
 *     block's sum of squares overflows fp32 (elements beyond about 2^58 in magnitude) the largest
 *     finite number is taken for it: the stored alpha_k, s_k are then not tau / sigma_k and its
 *     companion, but the codes and the ratio s_k / alpha_k, which is all decompression uses, are
 *     unaffected (the ablation modes without the post-rotation scale excepted: their codes depend
 *     on alpha_k).
 *     At the small end compression holds its accuracy down to blocks of bf16 subnormals
 *     (a block whose rotated maximum is below 2^-100 is scaled up by a power of two before
 *     Q_max / max|Z| is formed); decompression holds it down to elements of about 2^-112:
 *     below, the block factor s / (alpha sqrt(B)) is itself a subnormal fp32 number and the
 *     outputs are only within 2^-6 of the block's largest value
 *     (plus one bf16 subnormal step, 2^-133).
 *   - Return value: TACO_OK (0) or a negative taco_status.  Argument errors are found on
 *     the host before anything is launched.  TACO_ERR_LAUNCH is the result of this call's own
 *     launch; an error left on the thread by earlier, unrelated work is neither reported nor
 *     cleared.
 *   - A tensor has at most 2^36 elements (one launch covers it with one workgroup per 2048
 *     elements).
 */
#ifndef TACO_H_
#define TACO_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TACO_MAX_K 16               /* most payloads one taco_decompress_sum call can add        */
#define TACO_MAX_BATCH 32           /* most tensors one batched call can take                     */
#define TACO_MAX_BATCH_PAYLOADS 128 /* most payloads of all tensors of a batched decode together  */

typedef enum taco_status {
    TACO_OK = 0,
    TACO_ERR_NULL = -1,   /* a required pointer is NULL                               */
    TACO_ERR_SHAPE = -2,  /* rows <= 0, cols <= 0 or rows*cols above 2^36             */
    TACO_ERR_BLOCK = -3,  /* block is not one of 32, 64, 128, 256, 512                */
    TACO_ERR_ALIGN = -4,  /* a data pointer is not 16-byte aligned                    */
    TACO_ERR_K = -5,      /* k outside 1..TACO_MAX_K                                  */
    TACO_ERR_FORMAT = -6, /* params->format is not one of TACO_FORMAT_*               */
    TACO_ERR_LAUNCH = -7, /* the HIP runtime refused this call's launch               */
    TACO_ERR_IMPL = -8,   /* params->impl is not one of TACO_IMPL_*                   */
    TACO_ERR_PARAM = -9,  /* tau <= 0, eps < 0, or a non-finite parameter             */
    TACO_ERR_LAYOUT = -10,/* params->layout is not one of TACO_LAYOUT_*               */
    TACO_ERR_MODE = -11,  /* params->mode is outside 0..TACO_MODE_FULL                */
    TACO_ERR_OVERLAP = -12,/* an output buffer overlaps an input or another output    */
    TACO_ERR_BATCH = -13  /* count outside 1..TACO_MAX_BATCH, or count * k above
                             TACO_MAX_BATCH_PAYLOADS                                  */
} taco_status;

/* Code book.  E4M3 is the method's (chosen by the paper's format ablation, Section 5.3); E5M2
 * (OCP: bias 15, Q_max 57344) and INT8 (round(x / Delta), Delta = max|x| / 127, Section 2.3) are the
 * two alternatives that ablation compares against. */
enum { TACO_FORMAT_E4M3 = 0, TACO_FORMAT_E5M2 = 1, TACO_FORMAT_INT8 = 2 };

/* Stages of the method, for the paper's component ablations (Section 5.2.2, Section 5.3): a bit
 * mask.  Without RESCALE alpha_k = 1; without ROTATE Z_k = alpha_k G_k; without POSTSCALE s_k = 1
 * and Z_k itself is converted, saturating at +-Q_max.  FULL (7) is the method; 0 is the direct
 * cast, 4 dual scale only, 2 the standard Hadamard transform, 3 ASH without DS.  Every variant, with
 * any of the three code books, runs on either kernel family. */
enum { TACO_MODE_RESCALE = 1, TACO_MODE_ROTATE = 2, TACO_MODE_POSTSCALE = 4, TACO_MODE_FULL = 7 };

/* Kernel selection.  AUTO and MFMA run the matrix-core kernels (the rotation as a dense product on
 * the matrix cores; without the rotation, a product with the identity); BUTTERFLY runs the second
 * family, an in-register butterfly (kept for tests and benchmarks that compare the two).  Either
 * family handles any n, any mode and any code book in its one kernel. */
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

/* ---- Several tensors in one launch ------------------------------------------------------------
 * A launch costs a ramp-up and a drain of a few microseconds whatever it works on, which is a visible
 * share of the time for tensors of tens of megabytes (Section 4.4.1 counts kernel launches among the
 * costs that fusion removes; Section 4.4.2 exchanges the tensor in chunks of 64 MB).  The batched
 * calls run the same kernels over up to TACO_MAX_BATCH tensors (or chunks of one tensor: any row
 * range of a tensor whose element offset is a multiple of 2048 is a tensor of its own with its
 * pointers advanced) in ONE kernel.  All tensors of a call share `p`; the results are bit-identical
 * to the single calls.  The item arrays are HOST arrays, read during the call.
 * Errors: those of the single calls (the first offending item decides), TACO_ERR_BATCH for count
 * outside 1..TACO_MAX_BATCH or count * k above TACO_MAX_BATCH_PAYLOADS, and TACO_ERR_OVERLAP if an
 * output of one item overlaps an input or output of any item. */
typedef struct taco_compress_item {
    const void* x_bf16; /* in   device, rows*cols bf16 values                               */
    int64_t rows, cols;
    void* payload;      /* out  device, as for taco_compress                                */
    void* scales;       /* out  device, as for taco_compress (ignored when interleaved)     */
} taco_compress_item;

typedef struct taco_decode_item {
    const void* const* payloads; /* in   HOST array of k device pointers                    */
    const void* const* scales;   /* in   HOST array of k device pointers (or NULL when interleaved) */
    int64_t rows, cols;
    void* out_bf16;              /* out  device, rows*cols bf16 values                      */
} taco_decode_item;

int taco_compress_batch(const taco_compress_item* items, int32_t count, const taco_params* p, void* stream);

/* Every item adds k payloads (the same k for all items; k = 1 is taco_decompress). */
int taco_decompress_sum_batch(const taco_decode_item* items, int32_t count, int32_t k, const taco_params* p,
                              void* stream);

/* The fused decompress_sum -> compress of taco_decompress_sum_compress for several tensors (the chunks of one
 * exchange, or the shards one rank reduces for its peers) in ONE kernel; same k for all items. */
typedef struct taco_recompress_item {
    const void* const* payloads; /* in   HOST array of k device pointers                    */
    const void* const* scales;   /* in   HOST array of k device pointers (or NULL when interleaved) */
    int64_t rows, cols;
    void* payload_out;           /* out  device, taco_payload_bytes(n) (+ taco_scales_bytes(n) when interleaved) */
    void* scales_out;            /* out  device, taco_scales_bytes(n); ignored when interleaved */
} taco_recompress_item;

int taco_decompress_sum_compress_batch(const taco_recompress_item* items, int32_t count, int32_t k,
                                       const taco_params* p, void* stream);

/* Text for a taco_status value (static storage, never NULL). */
const char* taco_strerror(int status);

/* Library version, "major.minor". */
const char* taco_version(void);

/* Identifies the sources the library was built from: a hexadecimal digest of the kernel, host and
 * header files, fixed at compile time (static storage).  A build system or a benchmark can compare
 * it with the digest of the sources in front of it to detect a stale binary. */
const char* taco_build_id(void);

#ifdef __cplusplus
}
#endif
#endif /* TACO_H_ */
