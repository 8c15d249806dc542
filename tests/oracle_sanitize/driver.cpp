// Drives every entry point of the CPU oracle (oracle/taco_ref.cpp, compiled into this program with
// AddressSanitizer and UndefinedBehaviorSanitizer) over every block size, mode, code book and a set of
// ragged lengths.  Test infrastructure: it calls nothing but the oracle.  Exit status 0 = clean run.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <vector>

extern "C" {
int taco_ref_compress_ex(const void* x, int64_t n, int32_t block, float tau, float eps, int32_t mode, int32_t format, void* payload,
                         void* scales, void* z);
int taco_ref_decompress_sum_ex(const void* const* payloads, const void* const* scales, int32_t k, int64_t n, int32_t block,
                               int32_t mode, int32_t format, void* out, void* acc);
int taco_ref_hadamard_matrix(int32_t block, void* out);
int taco_ref_rotate(const void* x, int32_t block, void* y);
double taco_ref_format_decode(int32_t format, uint8_t code);
uint8_t taco_ref_format_encode(int32_t format, double v);
uint16_t taco_ref_float_to_bf16(float f);
}

static uint32_t rng_state = 12345u;
static float next_value() {              // small xorshift generator: values around zero with a few large ones
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 17; rng_state ^= rng_state << 5;
    const float u = static_cast<float>(rng_state & 0xFFFFFF) / 16777216.0f - 0.5f;
    return (rng_state >> 28) == 0 ? 40.0f * u : 0.05f * u;
}

int main() {
    const int blocks[] = {2, 8, 32, 64, 128, 256, 512};
    long runs = 0;
    for (int B : blocks) {
        std::vector<double> H(static_cast<size_t>(B) * B), v(B), w(B);
        if (taco_ref_hadamard_matrix(B, H.data()) != 0) return 10;
        for (int i = 0; i < B; ++i) v[i] = next_value();
        if (taco_ref_rotate(v.data(), B, w.data()) != 0) return 11;
        const int64_t lengths[] = {1, B - 1, B, B + 1, 5 * static_cast<int64_t>(B) + 3, 2048 + 77};
        for (int64_t n : lengths) {
            if (n < 1) continue;
            const int64_t M = (n + B - 1) / B;
            std::vector<uint16_t> x(n);
            for (auto& e : x) e = taco_ref_float_to_bf16(next_value());
            if (n > 4) { x[0] = 0; x[n / 2] = 0x8000; }                    // +0 and -0
            for (int mode = 0; mode < 8; ++mode) {
                for (int fmt = 0; fmt < 3; ++fmt) {
                    std::vector<uint8_t> p0(M * B), p1(M * B);
                    std::vector<float> s0(2 * M), s1(2 * M);
                    std::vector<double> z(M * B), acc(n);
                    std::vector<uint16_t> out(n);
                    if (taco_ref_compress_ex(x.data(), n, B, 1.0f, 1e-12f, mode, fmt, p0.data(), s0.data(), z.data()) != 0) return 12;
                    if (taco_ref_compress_ex(x.data(), n, B, 2.0f, 0.0f, mode, fmt, p1.data(), s1.data(), nullptr) != 0) return 13;
                    const void* pl[3] = {p0.data(), p1.data(), p0.data()};
                    const void* sc[3] = {s0.data(), s1.data(), s0.data()};
                    for (int k = 1; k <= 3; k += 2) {
                        if (taco_ref_decompress_sum_ex(pl, sc, k, n, B, mode, fmt, out.data(), acc.data()) != 0) return 14;
                        if (taco_ref_decompress_sum_ex(pl, sc, k, n, B, mode, fmt, out.data(), nullptr) != 0) return 15;
                    }
                    ++runs;
                }
            }
        }
    }
    for (int fmt = 0; fmt < 3; ++fmt)
        for (int c = 0; c < 256; ++c) {
            const double d = taco_ref_format_decode(fmt, static_cast<uint8_t>(c));
            if (std::isfinite(d)) (void)taco_ref_format_encode(fmt, d * 1.0001);
        }
    (void)taco_ref_format_encode(0, 1e300);
    (void)taco_ref_format_encode(1, -1e300);
    (void)taco_ref_format_encode(2, std::nan(""));
    // argument errors must be refused, not crash
    if (taco_ref_compress_ex(nullptr, 4, 128, 1.0f, 0.0f, 7, 0, nullptr, nullptr, nullptr) == 0) return 16;
    std::printf("oracle_sanitize: ok, %ld compress/decode combinations\n", runs);
    return 0;
}
