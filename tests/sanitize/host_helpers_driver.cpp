// Driver of the library's host-only entry points (quantizer parameters, multiplier encoding,
// weight preparation) for a build with the HOST code under -fsanitize=address,undefined
// (run by tests/test_sanitizers.py; no GPU call is made).  Prints "ok" and exits 0.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstring>
#include <limits>
#include <vector>

#include "qnn.h"

#define CHECK(cond)                                                             \
    do {                                                                        \
        if (!(cond)) {                                                          \
            std::fprintf(stderr, "check failed at line %d: %s\n", __LINE__, #cond); \
            return 1;                                                           \
        }                                                                       \
    } while (0)

int main()
{
    float s;
    int32_t z, lo, hi, m, sh;
    const double inf = std::numeric_limits<double>::infinity();
    CHECK(qnn_choose_qparams(2.1, 3.5, 8, &s, &z) == QNN_OK && z == 0);
    CHECK(qnn_choose_qparams(-1e300, 1e300, 8, &s, &z) == QNN_OK);
    CHECK(qnn_choose_qparams(-1e-320, 1e-320, 16, &s, &z) == QNN_OK);
    CHECK(qnn_choose_qparams(0.0, 0.0, 2, &s, &z) == QNN_OK && s == 1.0f);
    CHECK(qnn_choose_qparams(1.0, 0.0, 8, &s, &z) == QNN_EINVAL);
    CHECK(qnn_choose_qparams(std::nan(""), 0.0, 8, &s, &z) == QNN_EINVAL);
    CHECK(qnn_choose_qparams(0.0, 1.0, 8, nullptr, &z) == QNN_EINVAL);
    const double mults[] = {0.0, 1e-300, std::ldexp(1.0, -33), std::ldexp(1.0, -32), 0.5, 1.0 - std::ldexp(1.0, -40),
                            1.0, std::ldexp(1.0, 30), std::ldexp(1.0, 31) * 0.99};
    for (double v : mults) CHECK(qnn_quantize_multiplier(v, &m, &sh) == QNN_OK && sh >= -31 && sh <= 31);
    CHECK(qnn_quantize_multiplier(std::ldexp(1.0, 40), &m, &sh) == QNN_EINVAL);
    CHECK(qnn_quantize_multiplier(-1.0, &m, &sh) == QNN_EINVAL);
    CHECK(qnn_quantize_multiplier(inf, &m, &sh) == QNN_EINVAL);
    CHECK(qnn_act_range(2, 1e-30f, 3, &lo, &hi) == QNN_OK && hi == 255);
    CHECK(qnn_act_range(2, 1e30f, 3, &lo, &hi) == QNN_OK && hi == 3);
    CHECK(qnn_act_range(1, 0.1f, 255, &lo, &hi) == QNN_OK && lo == 255);
    CHECK(qnn_act_range(3, 0.1f, 0, &lo, &hi) == QNN_EINVAL);
    int32_t p[7];
    CHECK(qnn_qadd_params(0.02, 0.031, 0.04, &p[0], &p[1], &p[2], &p[3], &p[4], &p[5], &p[6]) == QNN_OK);
    (void)qnn_qadd_params(1e-30, 1e30, 1.0, &p[0], &p[1], &p[2], &p[3], &p[4], &p[5], &p[6]); // any status, no trap
    CHECK(qnn_qadd_params(0.0, 1.0, 1.0, &p[0], &p[1], &p[2], &p[3], &p[4], &p[5], &p[6]) == QNN_EINVAL);
    std::vector<float> w = {-1.0f, 0.5f, 3.4e38f, -3.4e38f, 0.0f, 1e-45f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
    std::vector<int8_t> wq(w.size());
    float d[2];
    for (int bits : {8, 4})
        for (int restricted : {0, 1}) CHECK(qnn_quantize_weights(w.data(), 2, 6, bits, restricted, wq.data(), d) == QNN_OK);
    CHECK(d[1] == 1.0f);
    std::vector<uint8_t> packed(w.size() / 2);
    CHECK(qnn_pack_int4(wq.data(), wq.size(), packed.data()) == QNN_OK);
    wq[3] = 8;
    CHECK(qnn_pack_int4(wq.data(), wq.size(), packed.data()) == QNN_EINVAL);
    CHECK(qnn_pack_int4(wq.data(), 3, packed.data()) == QNN_EINVAL);
    // argument validation of the device entry points returns before anything is launched
    CHECK(qnn_quantize(nullptr, nullptr, 4, 1.0f, 0, 0, 255, nullptr) == QNN_EINVAL);
    CHECK(std::strlen(qnn_version()) > 0);
    std::puts("ok");
    return 0;
}
