// Sanitizer run of the host-side code: the CPU oracle (oracle/fbq_oracle.c) and the library's host part
// (fbq_api.cpp: descriptor checks, fbq_pack, argument validation), built with -fsanitize=address,undefined
// and driven on small layers.  Checks, under the sanitizers: the oracle's pack/unpack round trip, the library's
// fbq_pack against the oracle's packer, the feedback bound |W - W_F| <= s/2 (Sec. 4.1), the oracle's linear
// against its own dense route, and the error paths of the entry points (nothing is ever launched: the kernel
// launchers are stubs).  Test infrastructure; prints "sanitize ok" when everything held.
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "fbq.h"

extern "C" {
double fbqo_half_to_double(uint16_t h);
uint16_t fbqo_double_to_half(double d);
int fbqo_quantize(int N, int K, int r, int bits, int group, const uint16_t *W, const uint16_t *A, const uint16_t *B,
                  uint8_t *codes, uint16_t *scales, uint16_t *zeros);
int fbqo_pack(int N, int K, int bits, const uint8_t *codes, uint32_t *words);
int fbqo_unpack(int N, int K, int bits, const uint32_t *words, uint8_t *codes);
int fbqo_reconstruct(int N, int K, int r, int bits, int group, const uint32_t *words, const uint16_t *scales,
                     const uint16_t *zeros, const uint16_t *A, const uint16_t *B, double *WF);
int fbqo_linear(int M, int N, int K, int r, int bits, int group, const uint16_t *x, const uint32_t *words,
                const uint16_t *scales, const uint16_t *zeros, const uint16_t *A, const uint16_t *B, double *y);
int fbqo_dense_linear(int M, int N, int K, const uint16_t *x, const double *Wd, double *y);
}

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static double uniform01()
{
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0;
}
static double normal() { return sqrt(-2.0 * log(uniform01() + 1e-300)) * cos(6.283185307179586 * uniform01()); }

#define REQUIRE(c) do { if (!(c)) { printf("FAILED: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

static int one_layer(int N, int K, int r, int bits, int M)
{
    const int G = K / 128, rw = K * bits / 32;
    std::vector<uint16_t> W((size_t)N * K), A((size_t)K * r), B((size_t)r * N), x((size_t)M * K), s((size_t)N * G), z((size_t)N * G);
    for (auto &v : W) v = fbqo_double_to_half(0.02 * normal() * (uniform01() < 0.01 ? 10.0 : 1.0));
    for (auto &v : A) v = fbqo_double_to_half(0.01 * normal());
    for (auto &v : B) v = fbqo_double_to_half(0.01 * normal());
    for (auto &v : x) v = fbqo_double_to_half(normal());
    std::vector<uint8_t> codes((size_t)N * K), back((size_t)N * K);
    std::vector<uint32_t> words((size_t)N * rw), words_lib((size_t)N * rw);
    REQUIRE(fbqo_quantize(N, K, r, bits, 128, W.data(), r ? A.data() : nullptr, r ? B.data() : nullptr, codes.data(), s.data(), z.data()) == 0);
    REQUIRE(fbqo_pack(N, K, bits, codes.data(), words.data()) == 0);
    REQUIRE(fbqo_unpack(N, K, bits, words.data(), back.data()) == 0);
    REQUIRE(memcmp(codes.data(), back.data(), codes.size()) == 0);

    // the library's host-side packer writes the same words, scales and zeros, and the transposed branch
    fbq_desc d = {N, K, r, bits, 128};
    std::vector<uint16_t> s_out(s.size()), z_out(z.size()), At((size_t)r * K), Bt((size_t)N * r);
    REQUIRE(fbq_packed_bytes(&d) == words.size() * 4);
    REQUIRE(fbq_pack(&d, codes.data(), s.data(), z.data(), r ? A.data() : nullptr, r ? B.data() : nullptr, words_lib.data(), s_out.data(),
                     z_out.data(), r ? At.data() : nullptr, r ? Bt.data() : nullptr) == FBQ_OK);
    REQUIRE(memcmp(words.data(), words_lib.data(), words.size() * 4) == 0);
    REQUIRE(s_out == s && z_out == z);
    for (int k = 0; k < K && r; k += 37)
        for (int j = 0; j < r; ++j) REQUIRE(At[(size_t)j * K + k] == A[(size_t)k * r + j]);
    for (int n = 0; n < N && r; n += 5)
        for (int j = 0; j < r; ++j) REQUIRE(Bt[(size_t)n * r + j] == B[(size_t)j * N + n]);
    codes[3] = (uint8_t)(1 << bits);                                // a code above qmax is refused
    REQUIRE(fbq_pack(&d, codes.data(), s.data(), z.data(), r ? A.data() : nullptr, r ? B.data() : nullptr, words_lib.data(), s_out.data(),
                     z_out.data(), r ? At.data() : nullptr, r ? Bt.data() : nullptr) == FBQ_ERR_SHAPE);

    // Sec. 4.1: |w - w_F| <= s/2 for every element
    std::vector<double> WF((size_t)N * K), y((size_t)M * N), y2((size_t)M * N);
    REQUIRE(fbqo_reconstruct(N, K, r, bits, 128, words.data(), s.data(), z.data(), r ? A.data() : nullptr, r ? B.data() : nullptr, WF.data()) == 0);
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k) {
            const double half_step = 0.5 * fbqo_half_to_double(s[(size_t)n * G + k / 128]);
            REQUIRE(fabs(fbqo_half_to_double(W[(size_t)n * K + k]) - WF[(size_t)n * K + k]) <= half_step * (1 + 1e-9));
        }
    // the fused formula against the dense product with W_F
    REQUIRE(fbqo_linear(M, N, K, r, bits, 128, x.data(), words.data(), s.data(), z.data(), r ? A.data() : nullptr, r ? B.data() : nullptr, y.data()) == 0);
    REQUIRE(fbqo_dense_linear(M, N, K, x.data(), WF.data(), y2.data()) == 0);
    double num = 0, den = 0;
    for (size_t i = 0; i < y.size(); ++i) { num += (y[i] - y2[i]) * (y[i] - y2[i]); den += y2[i] * y2[i]; }
    REQUIRE(sqrt(num / den) <= 1e-12);
    return 0;
}

int main()
{
    for (int bits = 3; bits <= 4; ++bits) {
        if (one_layer(9, 256, 16, bits, 3)) return 1;
        if (one_layer(5, 384, 0, bits, 1)) return 1;
        if (one_layer(33, 1408, 24, bits, 2)) return 1;
    }
    // entry points refuse bad arguments before anything is launched (pointers are never dereferenced)
    fbq_desc d = {16, 256, 8, 4, 128}, bad = {16, 200, 8, 4, 128};
    void *ok = (void *)0x1000, *odd = (void *)0x1004;
    REQUIRE(fbq_check_desc(&d) == FBQ_OK && fbq_check_desc(&bad) == FBQ_ERR_SHAPE && fbq_check_desc(nullptr) == FBQ_ERR_NULL);
    REQUIRE(fbq_workspace_bytes(&d, 1) > 0 && fbq_workspace_bytes(&bad, 1) == 0);
    REQUIRE(fbq_linear(&d, 1, nullptr, ok, ok, ok, ok, ok, ok, ok, 1 << 20, nullptr) == FBQ_ERR_NULL);
    REQUIRE(fbq_linear(&d, 1, odd, ok, ok, ok, ok, ok, ok, ok, 1 << 20, nullptr) == FBQ_ERR_ALIGN);
    REQUIRE(fbq_linear(&d, 1, ok, ok, ok, ok, ok, ok, ok, ok, 8, nullptr) == FBQ_ERR_WORKSPACE);
    REQUIRE(fbq_linear(&d, 0, ok, ok, ok, ok, ok, ok, ok, ok, 1 << 20, nullptr) == FBQ_ERR_SHAPE);
    fbq_layer_call calls[2];
    for (auto &c : calls) c = fbq_layer_call{d, ok, ok, ok, ok, ok, ok, ok, (void *)0x20000, fbq_workspace_bytes(&d, 1)};
    REQUIRE(fbq_linear_group(calls, 2, 1, nullptr) == FBQ_ERR_WORKSPACE);     // the same workspace twice
    REQUIRE(strcmp(fbq_status_string(FBQ_OK), "ok") == 0);
    printf("sanitize ok\n");
    return 0;
}
