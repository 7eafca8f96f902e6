// Host-side code of the library and the C oracle under AddressSanitizer and UndefinedBehaviorSanitizer: the packer,
// the pattern assignment, the connectivity selection, the export, the stride-2 parity form and the oracle's
// convolutions run on seeded layers, including ragged and degenerate ones.  Built and run by
// tests/test_host_sanitizers.py (g++ -fsanitize=address,undefined, runtimes linked statically); any report makes the
// process exit with a non-zero status.  The device side is replaced by the stubs at the end of this file: every
// handle is packed host-only.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "pconv.h"
#include "pconv_internal.h"

extern "C" {
int oracle_conv3x3(const float* x, const float* wm, const float* bias, int N, int C, int F, int H, int W, int stride,
                   int pad, int relu, double* y);
int oracle_conv3x3_at(const float* x, const float* wm, const float* bias, int N, int C, int F, int H, int W, int stride,
                      int pad, int relu, const int32_t* coords, long npts, double* out);
int oracle_maxpool2x2(const float* x, long planes, int H, int W, float* y);
}

namespace pconv {
int upload_packed(pconv_packed*) { return PCONV_EHIP; }
void release_device(pconv_packed*) {}
void set_hip_error(const char*, int) {}
}  // namespace pconv

static uint64_t g_state = 0x9E3779B97F4A7C15ull;
static double uniform01() {
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(g_state >> 11) / 9007199254740992.0;
}

#define CHECK(cond)                                                        \
    do {                                                                   \
        if (!(cond)) {                                                     \
            std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); \
            return 1;                                                      \
        }                                                                  \
    } while (0)

static int one_layer(int F, int C, int K, double keep, int dtype) {
    std::vector<uint16_t> lib;
    for (unsigned m = 0; m < 512 && (int)lib.size() < K; ++m)
        if (__builtin_popcount(m) == 4 && ((m >> 4) & 1u)) lib.push_back((uint16_t)m);
    CHECK((int)lib.size() == K);
    std::vector<float> w((size_t)F * C * 9);
    for (float& v : w) v = (float)(uniform01() - 0.5);
    std::vector<uint8_t> pid((size_t)F * C), mask((size_t)F * C);
    CHECK(pconv_assign_patterns(w.data(), F, C, lib.data(), K, pid.data()) == PCONV_OK);
    CHECK(pconv_select_connectivity(w.data(), F, C, lib.data(), K, pid.data(), keep, mask.data()) == PCONV_OK);
    std::vector<uint16_t> wh((size_t)F * C * 9);
    for (size_t i = 0; i < wh.size(); ++i) wh[i] = (uint16_t)(0x3000u + (i * 37u) % 0x0800u);   // finite fp16 patterns
    pconv_packed* p = nullptr;
    const void* wptr = dtype == PCONV_F16 ? (const void*)wh.data() : (const void*)w.data();
    CHECK(pconv_pack(wptr, dtype, F, C, lib.data(), K, pid.data(), mask.data(), PCONV_PACK_HOST_ONLY, &p) == PCONV_OK);
    size_t n_kept = 0;
    CHECK(pconv_packed_export(p, nullptr, nullptr, nullptr, nullptr, &n_kept) == PCONV_OK);
    std::vector<uint32_t> order((size_t)F), ptr((size_t)F * K + 1);
    std::vector<uint16_t> cin(n_kept + 1);
    std::vector<unsigned char> w4((n_kept + 1) * 4 * (dtype == PCONV_F16 ? 2 : 4));
    CHECK(pconv_packed_export(p, order.data(), ptr.data(), cin.data(), w4.data(), &n_kept) == PCONV_OK);
    CHECK(ptr[(size_t)F * K] == n_kept);
    int f2 = 0, c2 = 0, k2 = 0, d2 = 0;
    CHECK(pconv_packed_stats(p, &f2, &c2, &k2, &d2, &n_kept) == PCONV_OK && f2 == F && c2 == C && k2 == K && d2 == dtype);
    double mean = 0, mx = 0;
    (void)pconv_packed_balance(p, 16, 2, 1, &mean, &mx);
    for (int pad = 0; pad < 2; ++pad) {
        pconv_packed* q = nullptr;
        CHECK(pconv_packed_parity_form(p, pad, &q) == PCONV_OK);
        int kq = 0;
        CHECK(pconv_packed_stats(q, nullptr, nullptr, &kq, nullptr, nullptr) == PCONV_OK);
        std::vector<uint16_t> libq((size_t)kq + 1);
        CHECK(pconv_packed_library(q, libq.data()) == PCONV_OK);
        pconv_free(q);
    }
    pconv_free(p);
    return 0;
}

static int one_conv(int N, int C, int F, int H, int W, int stride, int pad) {
    std::vector<float> x((size_t)N * C * H * W), wm((size_t)F * C * 9), b((size_t)F);
    for (float& v : x) v = (float)uniform01();
    for (float& v : wm) v = uniform01() < 0.3 ? (float)(uniform01() - 0.5) : 0.f;
    for (float& v : b) v = (float)(uniform01() - 0.5);
    const int Ho = (H + 2 * pad - 3) / stride + 1, Wo = (W + 2 * pad - 3) / stride + 1;
    if (H + 2 * pad < 3 || W + 2 * pad < 3) return 0;
    std::vector<double> y((size_t)N * F * Ho * Wo);
    CHECK(oracle_conv3x3(x.data(), wm.data(), b.data(), N, C, F, H, W, stride, pad, 1, y.data()) == 0);
    std::vector<int32_t> coords = {0, 0, 0, 0, N - 1, F - 1, Ho - 1, Wo - 1};
    double at[2];
    CHECK(oracle_conv3x3_at(x.data(), wm.data(), b.data(), N, C, F, H, W, stride, pad, 1, coords.data(), 2, at) == 0);
    CHECK(at[0] == y[0] && at[1] == y[y.size() - 1]);
    if (H >= 2 && W >= 2) {
        std::vector<float> pooled((size_t)N * C * (H / 2) * (W / 2));
        CHECK(oracle_maxpool2x2(x.data(), (long)N * C, H, W, pooled.data()) == 0);
    }
    return 0;
}

int main() {
    static const int layers[][3] = {{1, 1, 1}, {3, 5, 4}, {17, 33, 8}, {64, 48, 12}, {130, 20, 56}, {40, 200, 8}};
    for (auto& l : layers)
        for (double keep : {0.0, 0.28, 1.0})
            for (int dtype : {PCONV_F32, PCONV_F16})
                if (one_layer(l[0], l[1], l[2], keep, dtype)) return 1;
    // argument errors take their exits
    uint16_t bad_lib[1] = {0x1FF};
    uint8_t pid1[1] = {0};
    float w9[9] = {0};
    if (pconv_assign_patterns(w9, 1, 1, bad_lib, 1, pid1) != PCONV_EPATTERN) return 1;
    if (pconv_assign_patterns(nullptr, 1, 1, bad_lib, 1, pid1) != PCONV_EINVAL) return 1;
    static const int convs[][7] = {{1, 1, 1, 1, 1, 1, 1}, {2, 3, 5, 4, 7, 1, 1}, {2, 5, 3, 9, 6, 2, 1}, {1, 4, 4, 8, 8, 2, 0},
                                   {3, 2, 7, 5, 13, 1, 0}, {1, 16, 8, 3, 3, 1, 0}};
    for (auto& c : convs)
        if (one_conv(c[0], c[1], c[2], c[3], c[4], c[5], c[6])) return 1;
    std::puts("host code and oracle clean under the sanitizers");
    return 0;
}
