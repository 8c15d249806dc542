// TACO reference ("oracle"): a plain, slow CPU statement of what the fused FP8
// compression operator computes.  TEST INFRASTRUCTURE ONLY: nothing on the product
// path may include, link or call this file; it shares no code with the HIP kernels.
//
// Every function follows one passage of the TACO paper (Section 4.2 "Adaptive
// Scale-Hadamard Transform", Section 4.3 "Dual-Scale FP8 Quantization", Algorithm 1):
//
//   partition      X = [G_1 .. G_M], contiguous blocks of B elements   (Eq. ash_partition)
//   sigma_k        sqrt( (1/B) sum_j G_kj^2 + eps )                     (Eq. ash_sigma)
//   alpha_k        tau / sigma_k                                        (Eq. ash_alpha)
//   Z_k            (1/sqrt(B)) H_B (alpha_k G_k)                        (Eq. ash_rotation)
//   s_k            max|Z_k| / Q_max                                     (Eq. post_scale)
//   q_k            Cvt_FP8( Z_k / s_k )                                 (Eq. quantization)
//   Zhat_k         Cvt_FP32(q_k) * s_k                                  (Eq. recon_dequant)
//   Ghat_k         (1/sqrt(B)) H_B Zhat_k                               (Eq. recon_ifwht)
//   G'_k           Ghat_k / alpha_k                                     (Eq. recon_rescale)
//
// Arithmetic is IEEE double.  A value is rounded to binary32 only where the method
// stores it (alpha_k and s_k travel as fp32 scalars beside the payload, Section 4.3
// "Dual-Scale Reconstruction"), and the stored value is what every later step reads.
// The rotation is the explicit B x B matrix product with
// H[i][j] = (-1)^popcount(i & j) (natural / Sylvester order); no fast transform, no
// blocking, no reordering.  OpenMP, when enabled, splits the loop over blocks only.
//
// Readings taken where the paper is silent (all listed in the design notes):
//   * FP8 is E4M3 in the OCP 8-bit floating point layout: 1 sign, 4 exponent (bias 7),
//     3 mantissa bits, subnormals, no infinities, S.1111.111 = NaN, Q_max = 448
//     (Section 5.3 format ablation selects E4M3; Section 2.3 gives the generic form).
//   * Cvt_FP8 rounds to nearest, ties to even, and saturates to +-448.
//   * A block whose rotated maximum is zero stores s_k = 0 and all-zero codes.
//   * The last block is zero padded when N is not a multiple of B; sigma still divides by B.
//   * The reduction of k decoded payloads accumulates in double, payload index ascending,
//     and rounds once to bf16 (via binary32), the one local reduction of Section 4.4.2.
//
// Ablation variants (Section 5.3 "Ablation Study", Section 5.2.2 "Component-wise Analysis"): the
// same pipeline with a stage switched off or another code book.  `mode` is a bit mask
//   1 rescale    alpha_k = tau / sigma_k, else alpha_k = 1           (Adaptive Scale)
//   2 rotate     Z_k = H (alpha G) / sqrt(B), else Z_k = alpha G     (Hadamard)
//   4 postscale  s_k = max|Z_k| / Q_max, else s_k = 1                (Dual-Scale)
// and `format` selects E4M3 (Q_max 448), E5M2 (Q_max 57344) or INT8 (round(x / Delta),
// Delta = max|x| / 127, Section 2.3).  mode 7 + E4M3 is the method itself; 0 is the direct cast,
// 4 "DS only", 2 the standard Hadamard transform, 3 ASH without DS.
//
// Pins: see tests/test_oracle_*.py (exhaustive E4M3 table against an independent
// library decode, H H^T = B I and a library Hadamard matrix, closed forms for the
// all-zero, single-outlier and constant blocks, brute-force scales, error bound).
// Parity unpinned: the paper prints no worked numeric example, so the choice of tau,
// eps, Hadamard ordering and payload layout is pinned only against this file.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <vector>
#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

constexpr double kQmax = 448.0;  // largest finite E4M3 magnitude (S.1111.110)

// ---- bf16 <-> double -------------------------------------------------------------------

double bf16_to_double(uint16_t h) {
    uint32_t u = static_cast<uint32_t>(h) << 16;
    float f;
    std::memcpy(&f, &u, sizeof f);
    return static_cast<double>(f);
}

// binary32 -> bf16, round to nearest, ties to even.  NaN keeps a quiet payload.
uint16_t float_to_bf16(float f) {
    uint32_t u;
    std::memcpy(&u, &f, sizeof u);
    if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<uint16_t>((u >> 16) | 0x0040u);
    uint32_t keep = u >> 16;
    uint32_t rest = u & 0xffffu;
    if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;
    return static_cast<uint16_t>(keep);
}

// ---- FP8 E4M3 ----------------------------------------------------------------------------

// Value of an 8-bit code  s eeee mmm :
//   e == 0          (m/8)      * 2^-6      (zero and subnormals, step 2^-9)
//   e == 15, m == 7 NaN
//   otherwise       (1 + m/8)  * 2^(e-7)
double e4m3_decode(uint8_t code) {
    int sign = code >> 7;
    int e = (code >> 3) & 0xf;
    int m = code & 0x7;
    double mag;
    if (e == 0xf && m == 0x7) return std::nan("");
    if (e == 0)
        mag = std::ldexp(static_cast<double>(m), -9);
    else
        mag = std::ldexp(8.0 + static_cast<double>(m), e - 10);
    return sign ? -mag : mag;
}

// Round an exact non-negative double to an integer, ties to the even integer.
double round_half_even(double v) {
    double fl = std::floor(v);
    double diff = v - fl;  // exact for the magnitudes used here (v < 2^10)
    if (diff > 0.5) return fl + 1.0;
    if (diff < 0.5) return fl;
    return (std::fmod(fl, 2.0) == 0.0) ? fl : fl + 1.0;
}

// Nearest E4M3 code, ties to even mantissa, saturating at +-448, sign kept on underflow.
uint8_t e4m3_encode(double v) {
    if (std::isnan(v)) return 0x7f;
    uint8_t sign = std::signbit(v) ? 0x80 : 0x00;
    double a = std::fabs(v);
    if (a >= kQmax) return sign | 0x7e;  // covers +-inf and every overshoot
    // Spacing of the grid around a: 2^-9 below 2^-6, else 2^(floor(log2 a) - 3).
    int ex;
    std::frexp(a, &ex);        // a = f * 2^ex, f in [0.5, 1)  =>  floor(log2 a) = ex - 1
    int p = (a < std::ldexp(1.0, -6)) ? -6 : ex - 1;
    double steps = round_half_even(std::ldexp(a, 3 - p));  // a in units of the local step
    // steps is in [0, 8] for subnormals, [8, 16] for normals; 16 carries into the next binade.
    int code;
    if (p == -6 && steps < 8.0) {
        code = static_cast<int>(steps);  // exponent field 0
    } else {
        if (steps == 16.0) { steps = 8.0; p += 1; }
        code = ((p + 7) << 3) | (static_cast<int>(steps) - 8);
    }
    if (code > 0x7e) code = 0x7e;
    return sign | static_cast<uint8_t>(code);
}

// ---- FP8 E5M2 (OCP): s eeeee mm, bias 15, subnormals (m/4) 2^-14, e = 31: infinity (m = 0) or NaN ----

constexpr double kQmaxE5M2 = 57344.0;   // 1.75 * 2^15

double e5m2_decode(uint8_t code) {
    int sign = code >> 7;
    int e = (code >> 2) & 0x1f;
    int m = code & 0x3;
    double mag;
    if (e == 0x1f) mag = (m == 0) ? INFINITY : std::nan("");
    else if (e == 0) mag = std::ldexp(static_cast<double>(m), -16);
    else mag = std::ldexp(4.0 + static_cast<double>(m), e - 17);
    return sign ? -mag : mag;
}

// Nearest E5M2 code, ties to even, saturating at +-57344, sign kept on underflow.
uint8_t e5m2_encode(double v) {
    if (std::isnan(v)) return 0x7f;
    uint8_t sign = std::signbit(v) ? 0x80 : 0x00;
    double a = std::fabs(v);
    if (a >= kQmaxE5M2) return sign | 0x7b;
    int ex;
    std::frexp(a, &ex);
    int p = (a < std::ldexp(1.0, -14)) ? -14 : ex - 1;
    double steps = round_half_even(std::ldexp(a, 2 - p));   // in units of the local step 2^(p-2)
    int code;
    if (p == -14 && steps < 4.0) {
        code = static_cast<int>(steps);
    } else {
        if (steps == 8.0) { steps = 4.0; p += 1; }
        code = ((p + 15) << 2) | (static_cast<int>(steps) - 4);
    }
    if (code > 0x7b) code = 0x7b;
    return sign | static_cast<uint8_t>(code);
}

// INT8 of Section 2.3: round to the nearest integer (ties to even), clamp to [-127, 127], two's complement byte.
uint8_t int8_encode(double v) {
    if (std::isnan(v)) return 0;
    double a = std::fabs(v);
    double r = a >= 127.0 ? 127.0 : round_half_even(a);
    int q = static_cast<int>(r);
    if (std::signbit(v)) q = -q;
    return static_cast<uint8_t>(static_cast<int8_t>(q));
}
double int8_decode(uint8_t code) { return static_cast<double>(static_cast<int8_t>(code)); }

enum { FORMAT_E4M3 = 0, FORMAT_E5M2 = 1, FORMAT_INT8 = 2 };
enum { MODE_RESCALE = 1, MODE_ROTATE = 2, MODE_POSTSCALE = 4, MODE_FULL = 7 };

double format_qmax(int format) { return format == FORMAT_E4M3 ? kQmax : format == FORMAT_E5M2 ? kQmaxE5M2 : 127.0; }
uint8_t format_encode(int format, double v) {
    return format == FORMAT_E4M3 ? e4m3_encode(v) : format == FORMAT_E5M2 ? e5m2_encode(v) : int8_encode(v);
}
double format_decode(int format, uint8_t c) {
    return format == FORMAT_E4M3 ? e4m3_decode(c) : format == FORMAT_E5M2 ? e5m2_decode(c) : int8_decode(c);
}

// ---- Hadamard matrix -----------------------------------------------------------------------

bool is_pow2(int64_t b) { return b >= 1 && (b & (b - 1)) == 0; }

int parity_of(unsigned v) {
    int p = 0;
    while (v) { p ^= 1; v &= v - 1; }
    return p;
}

// Row-major B x B matrix of +-1: H[i][j] = (-1)^popcount(i & j).
void fill_hadamard(int B, std::vector<double>& H) {
    H.resize(static_cast<size_t>(B) * B);
    for (int i = 0; i < B; ++i)
        for (int j = 0; j < B; ++j)
            H[static_cast<size_t>(i) * B + j] = parity_of(static_cast<unsigned>(i & j)) ? -1.0 : 1.0;
}

// y = H x (no normalisation), plain matrix-vector product.
void matvec(const std::vector<double>& H, int B, const double* x, double* y) {
    for (int i = 0; i < B; ++i) {
        const double* row = &H[static_cast<size_t>(i) * B];
        double acc = 0.0;
        for (int j = 0; j < B; ++j) acc += row[j] * x[j];
        y[i] = acc;
    }
}

// Decode one block of one payload into g'[0..B): Eqs. recon_dequant, recon_ifwht, recon_rescale.
void decode_block(const std::vector<double>& H, int B, const uint8_t* codes, float alpha_f,
                  float s_f, double* zhat, double* gprime, int mode = MODE_FULL, int format = FORMAT_E4M3) {
    const double alpha = static_cast<double>(alpha_f);
    const double s = static_cast<double>(s_f);
    const double root_b = std::sqrt(static_cast<double>(B));
    for (int i = 0; i < B; ++i) zhat[i] = format_decode(format, codes[i]) * s;
    if (mode & MODE_ROTATE) {
        matvec(H, B, zhat, gprime);
        for (int j = 0; j < B; ++j) gprime[j] = (gprime[j] / root_b) / alpha;
    } else {
        for (int j = 0; j < B; ++j) gprime[j] = zhat[j] / alpha;
    }
}

}  // namespace

extern "C" {

enum { TACO_REF_OK = 0, TACO_REF_ERR_ARG = -1 };

// Threads the block loops use (1 without OpenMP).
int taco_ref_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

// Sets the number of threads the block loops use from now on (no arithmetic depends on it: blocks are
// independent and each is computed by one thread); returns the number in effect.
int taco_ref_set_threads(int threads) {
#ifdef _OPENMP
    if (threads >= 1) omp_set_num_threads(threads);
    return omp_get_max_threads();
#else
    (void)threads;
    return 1;
#endif
}

double taco_ref_e4m3_decode(uint8_t code) { return e4m3_decode(code); }
double taco_ref_format_decode(int32_t format, uint8_t code) { return format_decode(format, code); }
uint8_t taco_ref_format_encode(int32_t format, double v) { return format_encode(format, v); }
uint8_t taco_ref_e4m3_encode(double v) { return e4m3_encode(v); }
uint16_t taco_ref_float_to_bf16(float f) { return float_to_bf16(f); }

// H (row-major, B*B doubles).
int taco_ref_hadamard_matrix(int32_t block, double* H_out) {
    if (!H_out || !is_pow2(block)) return TACO_REF_ERR_ARG;
    std::vector<double> H;
    fill_hadamard(block, H);
    std::memcpy(H_out, H.data(), H.size() * sizeof(double));
    return TACO_REF_OK;
}

// y = (1/sqrt(B)) H_B x : the orthonormal rotation of Eq. ash_rotation on one block.
int taco_ref_rotate(const double* x, int32_t block, double* y) {
    if (!x || !y || !is_pow2(block)) return TACO_REF_ERR_ARG;
    std::vector<double> H;
    fill_hadamard(block, H);
    matvec(H, block, x, y);
    const double root_b = std::sqrt(static_cast<double>(block));
    for (int i = 0; i < block; ++i) y[i] /= root_b;
    return TACO_REF_OK;
}

// Sender side of Algorithm 1.  x: n bf16 values (host).  payload: ceil(n/B)*B codes.
// scales: ceil(n/B) pairs {alpha_k, s_k} as fp32.  z_out (optional, may be null):
// ceil(n/B)*B doubles receiving the rotated values Z_k before quantisation.
// mode / format: ablation variants (see the header); MODE_FULL and FORMAT_E4M3 give the method.
int taco_ref_compress_ex(const uint16_t* x, int64_t n, int32_t block, float tau_f, float eps_f, int32_t mode,
                         int32_t format, uint8_t* payload, float* scales, double* z_out) {
    if (!x || !payload || !scales || n <= 0 || !is_pow2(block) || block < 2) return TACO_REF_ERR_ARG;
    if (mode < 0 || mode > MODE_FULL || format < FORMAT_E4M3 || format > FORMAT_INT8) return TACO_REF_ERR_ARG;
    const int B = block;
    const int64_t M = (n + B - 1) / B;
    const double tau = static_cast<double>(tau_f);
    const double eps = static_cast<double>(eps_f);
    const double root_b = std::sqrt(static_cast<double>(B));
    const double qmax = format_qmax(format);
    std::vector<double> H;
    fill_hadamard(B, H);

#pragma omp parallel
    {
        std::vector<double> g(B), w(B), z(B);
#pragma omp for schedule(static)
        for (int64_t k = 0; k < M; ++k) {
            // Eq. ash_partition: block k holds elements [kB, (k+1)B); zeros past n.
            for (int j = 0; j < B; ++j) {
                int64_t idx = k * B + j;
                g[j] = idx < n ? bf16_to_double(x[idx]) : 0.0;
            }
            // Eq. ash_sigma, Eq. ash_alpha.
            float alpha_f = 1.0f;
            if (mode & MODE_RESCALE) {
                double energy = 0.0;
                for (int j = 0; j < B; ++j) energy += g[j] * g[j];
                const double sigma = std::sqrt(energy / B + eps);
                alpha_f = static_cast<float>(tau / sigma);
            }
            const double alpha = static_cast<double>(alpha_f);
            // Rescale, then Eq. ash_rotation.
            for (int j = 0; j < B; ++j) g[j] = alpha * g[j];
            double amax = 0.0;
            if (mode & MODE_ROTATE) {
                matvec(H, B, g.data(), w.data());
                for (int i = 0; i < B; ++i) z[i] = w[i] / root_b;
            } else {
                for (int i = 0; i < B; ++i) z[i] = g[i];
            }
            for (int i = 0; i < B; ++i) amax = std::fmax(amax, std::fabs(z[i]));
            // Eq. post_scale, Eq. quantization.
            const float s_f = (mode & MODE_POSTSCALE) ? static_cast<float>(amax / qmax) : 1.0f;
            const double s = static_cast<double>(s_f);
            uint8_t* q = payload + k * B;
            for (int i = 0; i < B; ++i) q[i] = (s_f == 0.0f) ? 0x00 : format_encode(format, z[i] / s);
            scales[2 * k + 0] = alpha_f;
            scales[2 * k + 1] = s_f;
            if (z_out) std::memcpy(z_out + k * B, z.data(), sizeof(double) * B);
        }
    }
    return TACO_REF_OK;
}

int taco_ref_compress(const uint16_t* x, int64_t n, int32_t block, float tau_f, float eps_f,
                      uint8_t* payload, float* scales, double* z_out) {
    return taco_ref_compress_ex(x, n, block, tau_f, eps_f, MODE_FULL, FORMAT_E4M3, payload, scales, z_out);
}

// Receiver side of Algorithm 1 followed by the local reduction over k payloads:
// out[j] = bf16( fp32( sum_i G'^(i)_j ) ).  k = 1 is plain decompression.
// sum_out (optional): n doubles receiving the unrounded sum.
int taco_ref_decompress_sum_ex(const uint8_t* const* payloads, const float* const* scales, int32_t k,
                               int64_t n, int32_t block, int32_t mode, int32_t format, uint16_t* out,
                               double* sum_out) {
    if (!payloads || !scales || !out || k < 1 || n <= 0 || !is_pow2(block) || block < 2)
        return TACO_REF_ERR_ARG;
    if (mode < 0 || mode > MODE_FULL || format < FORMAT_E4M3 || format > FORMAT_INT8) return TACO_REF_ERR_ARG;
    for (int i = 0; i < k; ++i)
        if (!payloads[i] || !scales[i]) return TACO_REF_ERR_ARG;
    const int B = block;
    const int64_t M = (n + B - 1) / B;
    std::vector<double> H;
    fill_hadamard(B, H);

#pragma omp parallel
    {
        std::vector<double> zhat(B), gp(B), acc(B);
#pragma omp for schedule(static)
        for (int64_t b = 0; b < M; ++b) {
            for (int j = 0; j < B; ++j) acc[j] = 0.0;
            for (int i = 0; i < k; ++i) {
                decode_block(H, B, payloads[i] + b * B, scales[i][2 * b], scales[i][2 * b + 1],
                             zhat.data(), gp.data(), mode, format);
                for (int j = 0; j < B; ++j) acc[j] += gp[j];
            }
            for (int j = 0; j < B; ++j) {
                int64_t idx = b * B + j;
                if (idx >= n) break;
                if (sum_out) sum_out[idx] = acc[j];
                out[idx] = float_to_bf16(static_cast<float>(acc[j]));
            }
        }
    }
    return TACO_REF_OK;
}

int taco_ref_decompress_sum(const uint8_t* const* payloads, const float* const* scales, int32_t k,
                            int64_t n, int32_t block, uint16_t* out, double* sum_out) {
    return taco_ref_decompress_sum_ex(payloads, scales, k, n, block, MODE_FULL, FORMAT_E4M3, out, sum_out);
}

int taco_ref_decompress(const uint8_t* payload, const float* scales, int64_t n, int32_t block,
                        uint16_t* out, double* sum_out) {
    const uint8_t* p[1] = {payload};
    const float* s[1] = {scales};
    return taco_ref_decompress_sum(p, s, 1, n, block, out, sum_out);
}

}  // extern "C"
