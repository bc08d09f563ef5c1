// Host self test, meant for a build of the library's host sources with AddressSanitizer and UBSan (no GPU needed):
// the layout transforms (lqer_selftest_layouts), the argument checks of the C ABI, and the offline step's host
// arithmetic for every format (on a machine without a GPU the final upload fails with LQER_ERR_HIP, after all of the
// host work has run under the sanitizers; with a GPU it succeeds).
#include <cmath>
#include <cstdio>
#include <vector>

#include "lqer.h"

static int fails = 0;
static void expect(bool ok, const char* what) {
    if (!ok) { std::printf("FAIL: %s\n", what); ++fails; }
}

int main() {
    expect(lqer_selftest_layouts() == LQER_OK, "layout round trip");
    lqer_layer* h = nullptr;
    uint8_t wc[128] = {0}, we[8] = {0};
    expect(lqer_layer_import(100, 10, 0, wc, we, nullptr, nullptr, nullptr, nullptr, &h) == LQER_ERR_SHAPE, "K % 16");
    expect(lqer_layer_import_w(3, 16, 16, 0, wc, we, nullptr, nullptr, nullptr, nullptr, &h) == LQER_ERR_UNSUPPORTED, "w_bits");
    expect(lqer_int_layer_import(192, 16, 0, wc, (const uint16_t*)we, nullptr, nullptr, nullptr, nullptr, &h) == LQER_ERR_SHAPE, "K % 128");
    expect(lqer_linear_workspace_bytes(nullptr, 4) == 0, "null layer");
    uint64_t st = 12345;
    auto rnd = [&st]() { st = st * 6364136223846793005ull + 1442695040888963407ull; return (double)(st >> 40) / (double)(1 << 24) - 0.5; };
    const int64_t K = 256, N = 48;
    std::vector<float> W((size_t)K * N), calib((size_t)2 * 8 * K);
    for (auto& v : W) v = (float)(0.04 * rnd());
    for (auto& v : calib) v = (float)(std::fabs(rnd()) + 0.1);
    const lqer_config cfgs[] = {{4, 8, 8, 16}, {4, 8, 4, 16}, {2, 8, 8, 16}, {4, 8, 16, 128}};
    for (const auto& c : cfgs)
        for (int k : {0, 8, 40}) {
            h = nullptr;
            const int s = lqer_build_factors(W.data(), K, N, calib.data(), 2, 8, k, 1, &c, &h);
            expect(s == LQER_OK || s == LQER_ERR_HIP, "lqer_build_factors status");
            if (s == LQER_OK) lqer_layer_free(h);
        }
    const lqer_config bad = {5, 8, 8, 16};
    expect(lqer_build_factors(W.data(), K, N, calib.data(), 2, 8, 8, 1, &bad, &h) == LQER_ERR_UNSUPPORTED, "bad config");
    std::printf(fails ? "host self test: %d failure(s)\n" : "host self test ok\n", fails);
    return fails ? 1 : 0;
}
