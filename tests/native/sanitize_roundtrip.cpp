// Host-code sanitizer pass: the offline packer (lqq_pack.cpp) and the C oracle (lqq_oracle.c)
// built with -fsanitize=address,undefined and driven through a pack / unpack / dequantise /
// multiply round trip, including ragged thread splits and the error paths.  Any out-of-bounds
// access, misaligned access or signed overflow aborts the program; a wrong value exits non-zero.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "liquidgemm.h"

extern "C" {
int lqq_oracle_dequant(int N, int K, int g, const uint8_t *packed, const uint8_t *s_u8, const uint8_t *a,
                       int8_t *Wd);
int lqq_oracle_w4a8_gemm(int M, int N, int K, int g, const int8_t *X, const float *s_x, const uint8_t *packed,
                         const uint8_t *s_u8, const uint8_t *a, const float *s_w, int32_t *ACC, double *Y);
}

static uint32_t g_state = 12345u;
static uint32_t next_u32()
{
    g_state = g_state * 1664525u + 1013904223u;
    return g_state >> 8;
}

#define REQUIRE(cond)                                                         \
    do {                                                                      \
        if (!(cond)) {                                                        \
            std::fprintf(stderr, "%s:%d: %s failed\n", __FILE__, __LINE__, #cond); \
            std::exit(1);                                                     \
        }                                                                     \
    } while (0)

static void round_trip(int N, int K, int g, int M)
{
    size_t cb = 0, gb = 0;
    REQUIRE(liquidquant_packed_size(N, K, g, &cb, &gb) == LQ_OK);
    REQUIRE(cb == (size_t)N * K / 2 && gb == (size_t)2 * N * K / g);
    const int G = K / g;
    // exactly sized heap buffers: the sanitizer sees any byte past their ends
    std::vector<int8_t> Q((size_t)N * K);
    for (auto &q : Q) q = (int8_t)((int)(next_u32() % 239u) - 119);
    std::vector<uint8_t> packed(cb), gparams(gb);
    REQUIRE(liquidquant_pack_from_i8(Q.data(), N, K, g, packed.data(), gparams.data()) == LQ_OK);
    std::vector<uint8_t> codes((size_t)N * K), s_u8((size_t)N * G), a((size_t)N * G);
    REQUIRE(liquidquant_unpack_weights(packed.data(), gparams.data(), N, K, g, codes.data(), s_u8.data(), a.data()) == LQ_OK);
    // canonical form of the oracle: two codes per byte, even k in the low nibble
    std::vector<uint8_t> canon((size_t)N * K / 2);
    for (size_t i = 0; i < canon.size(); ++i) {
        REQUIRE(codes[2 * i] <= 15 && codes[2 * i + 1] <= 15);
        canon[i] = (uint8_t)(codes[2 * i] | (codes[2 * i + 1] << 4));
    }
    std::vector<int8_t> Wd((size_t)N * K);
    REQUIRE(lqq_oracle_dequant(N, K, g, canon.data(), s_u8.data(), a.data(), Wd.data()) == 0);
    for (size_t i = 0; i < Wd.size(); ++i) {  // reconstruction bound of the two-level scheme
        const int d = (int)Wd[i] - (int)Q[i];
        REQUIRE(d >= -8 && d <= 8);
    }
    // the float entry points on weights that quantise back to Q (scale 1: amax = 119)
    std::vector<float> W((size_t)N * K), s_w(N);
    std::vector<uint16_t> W16((size_t)N * K);
    for (int n = 0; n < N; ++n) {
        Q[(size_t)n * K] = 119;
        for (int k = 0; k < K; ++k) W[(size_t)n * K + k] = (float)Q[(size_t)n * K + k];
    }
    std::vector<uint8_t> packed2(cb), gparams2(gb);
    REQUIRE(liquidquant_pack_weights(W.data(), N, K, g, packed2.data(), gparams2.data(), s_w.data()) == LQ_OK);
    REQUIRE(liquidquant_pack_from_i8(Q.data(), N, K, g, packed.data(), gparams.data()) == LQ_OK);
    REQUIRE(packed == packed2 && gparams == gparams2);
    for (int n = 0; n < N; ++n) REQUIRE(s_w[n] == 1.0f);
    for (auto &h : W16) h = 0x3C00;  // 1.0 in binary16
    REQUIRE(liquidquant_pack_weights_f16(W16.data(), N, K, g, packed2.data(), gparams2.data(), s_w.data()) == LQ_OK);
    // whole oracle path against a plain triple loop on the dequantised matrix
    REQUIRE(liquidquant_unpack_weights(packed.data(), gparams.data(), N, K, g, codes.data(), s_u8.data(), a.data()) == LQ_OK);
    for (size_t i = 0; i < canon.size(); ++i) canon[i] = (uint8_t)(codes[2 * i] | (codes[2 * i + 1] << 4));
    REQUIRE(lqq_oracle_dequant(N, K, g, canon.data(), s_u8.data(), a.data(), Wd.data()) == 0);
    std::vector<int8_t> X((size_t)M * K);
    for (auto &x : X) x = (int8_t)((int)(next_u32() % 255u) - 127);
    std::vector<float> s_x(M, 0.5f);
    std::vector<int32_t> ACC((size_t)M * N);
    std::vector<double> Y((size_t)M * N);
    REQUIRE(lqq_oracle_w4a8_gemm(M, N, K, g, X.data(), s_x.data(), canon.data(), s_u8.data(), a.data(), s_w.data(),
                                 ACC.data(), Y.data()) == 0);
    for (int m = 0; m < M; ++m)
        for (int n = 0; n < N; ++n) {
            long long acc = 0;
            for (int k = 0; k < K; ++k) acc += (long long)X[(size_t)m * K + k] * Wd[(size_t)n * K + k];
            REQUIRE(ACC[(size_t)m * N + n] == acc);
        }
}

int main()
{
    round_trip(64, 256, 64, 3);
    round_trip(64, 256, 128, 1);
    round_trip(192, 768, 64, 5);    // three thread shares of 64 rows
    round_trip(1088, 512, 128, 2);  // ragged split of the rows over the packer's threads
    // error paths: nothing may be touched
    size_t cb, gb;
    REQUIRE(liquidquant_packed_size(63, 256, 64, &cb, &gb) == LQ_ERR_INVALID);
    REQUIRE(liquidquant_packed_size(64, 250, 64, &cb, &gb) == LQ_ERR_INVALID);
    REQUIRE(liquidquant_packed_size(64, 256, 32, &cb, &gb) == LQ_ERR_INVALID);
    REQUIRE(liquidquant_packed_size(64, 256, 64, nullptr, nullptr) == LQ_OK);
    std::vector<int8_t> bad((size_t)64 * 256, (int8_t)120);  // beyond the protective range
    std::vector<uint8_t> p((size_t)64 * 128), gpar((size_t)2 * 64 * 4);
    REQUIRE(liquidquant_pack_from_i8(bad.data(), 64, 256, 64, p.data(), gpar.data()) == LQ_ERR_INVALID);
    REQUIRE(liquidquant_pack_from_i8(nullptr, 64, 256, 64, p.data(), gpar.data()) == LQ_ERR_INVALID);
    REQUIRE(w4a8_last_error()[0] != 0);
    // the oracle rejects triples that violate Eq. 11 instead of wrapping
    std::vector<uint8_t> canon((size_t)64 * 128, 0xFF), s((size_t)64 * 4, 16), off((size_t)64 * 4, 200);
    std::vector<int8_t> Wd((size_t)64 * 256);
    REQUIRE(lqq_oracle_dequant(64, 256, 64, canon.data(), s.data(), off.data(), Wd.data()) != 0);
    std::puts("sanitize_roundtrip ok");
    return 0;
}
