// Offline LiquidQuant packer (host code): two-level quantisation of Sec. 4 of the paper
// followed by the permutation into the gfx950 operand order described in lqq_layout.h.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <thread>
#include <vector>

#include "lqq_common.h"
#include "lqq_layout.h"

namespace lqq {

static thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

const char *last_error() { return g_err; }

namespace {

// Runs fn(row_begin, row_end) over [0, rows) on a few host threads.
template <class Fn>
void parallel_rows(int rows, Fn fn)
{
    unsigned hw = std::thread::hardware_concurrency();
    int nt = (int)std::min<unsigned>(hw ? hw : 1, 16);
    nt = std::max(1, std::min(nt, rows / 64));
    if (nt == 1) {
        fn(0, rows);
        return;
    }
    std::vector<std::thread> th;
    const int per = (rows + nt - 1) / nt;
    for (int i = 0; i < nt; ++i) {
        const int b = i * per, e = std::min(rows, b + per);
        if (b < e) th.emplace_back([=] { fn(b, e); });
    }
    for (auto &t : th) t.join();
}

float half_bits_to_float(uint16_t h)
{
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    const uint32_t exp = (h >> 10) & 0x1Fu;
    uint32_t man = h & 0x3FFu;
    uint32_t bits;
    if (exp == 0) {
        if (man == 0) {
            bits = sign;
        } else {  // subnormal: renormalise
            int e = -1;
            do {
                ++e;
                man <<= 1;
            } while (!(man & 0x400u));
            bits = sign | ((uint32_t)(127 - 15 - e) << 23) | ((man & 0x3FFu) << 13);
        }
    } else if (exp == 31) {
        bits = sign | 0x7F800000u | (man << 13);
    } else {
        bits = sign | ((exp + 127 - 15) << 23) | (man << 13);
    }
    float f;
    std::memcpy(&f, &bits, 4);
    return f;
}

// Level 2 of one channel (Eq. 7, Eq. 10) and scatter into the packed blob.
// q: the channel's K level-1 integers, all in [-119, 119].
void pack_channel(const int8_t *q, int n, int K, int group, uint8_t *codes, uint8_t *gparams)
{
    const int G = K / group;
    for (int gi = 0; gi < G; ++gi) {
        const int8_t *qg = q + (size_t)gi * group;
        int mn = qg[0], mx = qg[0];
        for (int i = 1; i < group; ++i) {
            mn = std::min<int>(mn, qg[i]);
            mx = std::max<int>(mx, qg[i]);
        }
        const int R = mx - mn;                        // max(Q_u8)
        const int s = std::max(1, (2 * R + 15) / 30); // round(R / 15); no tie since 15 is odd
        const size_t pl = gparam_loc(n, gi, K, group);
        gparams[pl] = (uint8_t)s;
        gparams[pl + 1] = (uint8_t)(128 + mn);        // a = 2^7 + min(Q_i8)
        for (int i = 0; i < group; ++i) {
            const int qu = qg[i] - mn;                // Q_u8
            const int code = std::min(15, (2 * qu + s) / (2 * s));  // round half up, clamp
            const CodeLoc cl = code_loc(n, gi * group + i, K);
            codes[cl.byte] = (uint8_t)(codes[cl.byte] | (code << cl.shift));
        }
    }
}

int check_pack_args(const void *src, int N, int K, int group, const void *W_packed,
                    const void *gparams)
{
    if (!shape_ok(N, K, group))
        return fail(LQ_ERR_INVALID,
                    "bad shape N=%d K=%d group=%d (need N%%64==0, K%%256==0, group 64|128, K<=131072)",
                    N, K, group);
    if (!src || !W_packed || !gparams) return fail(LQ_ERR_INVALID, "null pointer");
    return LQ_OK;
}

template <class LoadRow>
int pack_float_rows(LoadRow load_row, int N, int K, int group, void *W_packed, uint8_t *gparams,
                    float *w_scales)
{
    uint8_t *codes = static_cast<uint8_t *>(W_packed);
    std::memset(codes, 0, (size_t)N * K / 2);
    // The two nibbles of a byte belong to the same channel, so distinct channels never
    // touch the same byte and rows can be packed concurrently.
    parallel_rows(N, [&](int nb, int ne) {
        std::vector<float> w(K);
        std::vector<int8_t> q(K);
        for (int n = nb; n < ne; ++n) {
            load_row(n, w.data());
            float amax = 0.0f;
            for (int k = 0; k < K; ++k) amax = std::max(amax, std::fabs(w[k]));
            // Level 1 (Sec. 4, Eq. 1 with z = 0 and the protective range [-119, 119]).
            const float s_w = amax > 0.0f ? amax / 119.0f : 1.0f;
            w_scales[n] = s_w;
            for (int k = 0; k < K; ++k) {
                float r = std::nearbyintf(w[k] / s_w);  // FP32 quotient, round half to even
                r = std::min(119.0f, std::max(-119.0f, r));
                q[k] = (int8_t)r;
            }
            pack_channel(q.data(), n, K, group, codes, gparams);
        }
    });
    return LQ_OK;
}

}  // namespace
}  // namespace lqq

using namespace lqq;

extern "C" {

int w4a8_version(void) { return 2; }

const char *w4a8_last_error(void) { return lqq::last_error(); }

int liquidquant_packed_size(int N, int K, int group, size_t *codes_bytes, size_t *gparams_bytes)
{
    if (!shape_ok(N, K, group)) return fail(LQ_ERR_INVALID, "bad shape N=%d K=%d group=%d", N, K, group);
    if (codes_bytes) *codes_bytes = (size_t)N * K / 2;
    if (gparams_bytes) *gparams_bytes = (size_t)N * (K / group) * 2;
    return LQ_OK;
}

int liquidquant_pack_weights(const float *W, int N, int K, int group, void *W_packed,
                             uint8_t *gparams, float *w_scales)
{
    if (int rc = check_pack_args(W, N, K, group, W_packed, gparams)) return rc;
    if (!w_scales) return fail(LQ_ERR_INVALID, "null w_scales");
    for (size_t i = 0, e = (size_t)N * K; i < e; ++i)
        if (!std::isfinite(W[i])) return fail(LQ_ERR_INVALID, "W[%zu] is not finite", i);
    return pack_float_rows(
        [&](int n, float *dst) { std::memcpy(dst, W + (size_t)n * K, sizeof(float) * K); }, N, K,
        group, W_packed, gparams, w_scales);
}

int liquidquant_pack_weights_f16(const uint16_t *W_f16, int N, int K, int group, void *W_packed,
                                 uint8_t *gparams, float *w_scales)
{
    if (int rc = check_pack_args(W_f16, N, K, group, W_packed, gparams)) return rc;
    if (!w_scales) return fail(LQ_ERR_INVALID, "null w_scales");
    for (size_t i = 0, e = (size_t)N * K; i < e; ++i)
        if ((W_f16[i] & 0x7C00u) == 0x7C00u) return fail(LQ_ERR_INVALID, "W[%zu] is not finite", i);
    return pack_float_rows(
        [&](int n, float *dst) {
            const uint16_t *src = W_f16 + (size_t)n * K;
            for (int k = 0; k < K; ++k) dst[k] = half_bits_to_float(src[k]);
        },
        N, K, group, W_packed, gparams, w_scales);
}

int liquidquant_pack_from_i8(const int8_t *Q_i8, int N, int K, int group, void *W_packed,
                             uint8_t *gparams)
{
    if (int rc = check_pack_args(Q_i8, N, K, group, W_packed, gparams)) return rc;
    for (size_t i = 0, e = (size_t)N * K; i < e; ++i)
        if (Q_i8[i] < -119 || Q_i8[i] > 119)
            return fail(LQ_ERR_INVALID, "Q_i8[%zu] = %d outside the protective range [-119, 119]", i,
                        (int)Q_i8[i]);
    uint8_t *codes = static_cast<uint8_t *>(W_packed);
    std::memset(codes, 0, (size_t)N * K / 2);
    parallel_rows(N, [&](int nb, int ne) {
        for (int n = nb; n < ne; ++n) pack_channel(Q_i8 + (size_t)n * K, n, K, group, codes, gparams);
    });
    return LQ_OK;
}

int liquidquant_unpack_weights(const void *W_packed, const uint8_t *gparams, int N, int K,
                               int group, uint8_t *codes, uint8_t *s_u8, uint8_t *a)
{
    if (int rc = check_pack_args(W_packed, N, K, group, W_packed, gparams)) return rc;
    const uint8_t *blob = static_cast<const uint8_t *>(W_packed);
    const int G = K / group;
    parallel_rows(N, [&](int nb, int ne) {
        for (int n = nb; n < ne; ++n) {
            if (codes)
                for (int k = 0; k < K; ++k) {
                    const CodeLoc cl = code_loc(n, k, K);
                    codes[(size_t)n * K + k] = (uint8_t)((blob[cl.byte] >> cl.shift) & 0x0F);
                }
            for (int gi = 0; gi < G; ++gi) {
                const size_t pl = gparam_loc(n, gi, K, group);
                if (s_u8) s_u8[(size_t)n * G + gi] = gparams[pl];
                if (a) a[(size_t)n * G + gi] = gparams[pl + 1];
            }
        }
    });
    return LQ_OK;
}

// W8A8 reference (Sec. 3.2 / 7.3: the no-dequantisation baseline): INT8 weights in the order in
// which the reference kernel's lanes consume them.  Per tile of 32 channels and k-step of
// 32: 64 lanes x 16 bytes, lane = 32 * kb + j holding W[n][32 step + 16 kb + 0..15] with
// n = 64 (tile / 2) + 2 j + tile % 2: as in the 4-bit layout, the two tiles of a wave
// interleave their channels so that a lane stores two adjacent outputs.
int w8a8_pack_weights(const int8_t *W_i8, int N, int K, void *W8_packed)
{
    if (!shape_ok(N, K, 64)) return fail(LQ_ERR_INVALID, "bad shape N=%d K=%d", N, K);
    if (!W_i8 || !W8_packed) return fail(LQ_ERR_INVALID, "null pointer");
    int8_t *out = static_cast<int8_t *>(W8_packed);
    const int steps = K / 32;
    parallel_rows(N / 32, [&](int tb, int te) {
        for (int tile = tb; tile < te; ++tile)
            for (int st = 0; st < steps; ++st)
                for (int lane = 0; lane < 64; ++lane) {
                    const int j = lane & 31, kb = lane >> 5;
                    std::memcpy(out + (((size_t)tile * steps + st) * 64 + lane) * 16,
                                W_i8 + (size_t)(64 * (tile >> 1) + 2 * j + (tile & 1)) * K + 32 * st + 16 * kb, 16);
                }
    });
    return LQ_OK;
}

}  // extern "C"
