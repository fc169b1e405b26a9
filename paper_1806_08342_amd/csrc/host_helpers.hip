// Host-only entry points of the C ABI: quantizer parameter selection, fixed-point
// multiplier encoding, weight preparation.  No GPU work happens here.
#include <cmath>
#include <cstdio>
#include <cstring>
#include <limits>

#include <cstdlib>

#include "qnn_device.h"
#include "tuning.h"

namespace qnn {

static thread_local char g_last_error[256] = "";

qnn_status launch_status(hipError_t e)
{
    if (e == hipSuccess) return QNN_OK;
    std::snprintf(g_last_error, sizeof(g_last_error), "%s: %s", hipGetErrorName(e), hipGetErrorString(e));
    return QNN_ELAUNCH;
}

struct TuningField {
    const char *name;
    int Tuning::*field;
    int unset;
};
static const TuningField kTuningFields[] = {
    {"QNN_FORCE_SPLIT", &Tuning::force_split, 0}, {"QNN_NO_SHORTK", &Tuning::no_shortk, 0},
    {"QNN_BRES", &Tuning::bres, -1},              {"QNN_STEM_BLOCK", &Tuning::stem_block, 0},
    {"QNN_XCD_ROWS", &Tuning::xcd_rows, -1},      {"QNN_DW_RH", &Tuning::dw_rh, 0},
    {"QNN_DW_MAD", &Tuning::dw_mad, 0},           {"QNN_GEMM_PRIO", &Tuning::gemm_prio, -1},
    {"QNN_PERSIST", &Tuning::persist, -1},        {"QNN_DW_VARIANT", &Tuning::dw_variant, -1},
    {"QNN_DW_XCD", &Tuning::dw_xcd, 1},
    {"QNN_SHORTK_ALDS", &Tuning::shortk_alds, 1},
};

static bool tuning_assign(Tuning &t, const char *name, const char *value)
{
    if (std::strcmp(name, "QNN_FORCE_TILE") == 0) {
        std::snprintf(t.force_tile, sizeof t.force_tile, "%s", value ? value : "");
        return true;
    }
    for (const TuningField &f : kTuningFields)
        if (std::strcmp(name, f.name) == 0) {
            // a switch that is set without a number counts as 1, as the bare environment variable did
            t.*(f.field) = value ? ((*value == 0) ? 1 : std::atoi(value)) : f.unset;
            return true;
        }
    return false;
}

Tuning &tuning()
{
    static Tuning t = [] {
        Tuning init;
        (void)tuning_assign(init, "QNN_FORCE_TILE", std::getenv("QNN_FORCE_TILE"));
        for (const TuningField &f : kTuningFields) (void)tuning_assign(init, f.name, std::getenv(f.name));
        return init;
    }();
    return t;
}

void set_last_error(const char *text) { std::snprintf(g_last_error, sizeof(g_last_error), "%s", text); }

// nearest integer, halves go away from zero
static double nearest_away(double v) { return std::copysign(std::floor(std::fabs(v) + 0.5), v); }

} // namespace qnn

extern "C" {

const char *qnn_last_error(void) { return qnn::g_last_error; }

const char *qnn_version(void) { return "0.2"; }

qnn_status qnn_tuning_set(const char *name, const char *value)
{
    if (!name) return QNN_EINVAL;
    return qnn::tuning_assign(qnn::tuning(), name, value) ? QNN_OK : QNN_EINVAL;
}

// Sec. 2.1: the range is widened to hold 0 so that real 0 maps to the integer z exactly.
qnn_status qnn_choose_qparams(double xmin, double xmax, int bits, float *scale, int32_t *zero_point)
{
    if (scale == nullptr || zero_point == nullptr || bits < 2 || bits > 16) return QNN_EINVAL;
    if (std::isnan(xmin) || std::isnan(xmax) || xmin > xmax) return QNN_EINVAL;
    const double lo = std::fmin(xmin, 0.0), hi = std::fmax(xmax, 0.0);
    const double steps = std::ldexp(1.0, bits) - 1.0;
    if (hi - lo == 0.0) {
        *scale = 1.0f;
        *zero_point = 0;
        return QNN_OK;
    }
    const float s = static_cast<float>((hi - lo) / steps);
    double z = qnn::nearest_away(-lo / static_cast<double>(s));
    z = std::fmin(std::fmax(z, 0.0), steps);
    *scale = s;
    *zero_point = static_cast<int32_t>(z);
    return QNN_OK;
}

qnn_status qnn_quantize_multiplier(double real_mult, int32_t *mult, int32_t *shift)
{
    if (mult == nullptr || shift == nullptr || !(real_mult >= 0.0) || std::isinf(real_mult)) return QNN_EINVAL;
    *mult = 0;
    *shift = 0;
    if (real_mult == 0.0) return QNN_OK;
    int exponent = 0;
    const double mant = std::frexp(real_mult, &exponent); // [0.5, 1)
    long long fixed = std::llround(std::ldexp(mant, 31));
    if (fixed >= (1ll << 31)) { // mantissa rounded up to 1.0
        fixed = 1ll << 30;
        exponent += 1;
    }
    if (exponent < -31) return QNN_OK;     // below 2^-32: rescales every int32 to 0
    if (exponent > 31) return QNN_EINVAL;  // would need a left shift of more than 31
    *mult = static_cast<int32_t>(fixed);
    *shift = -exponent;
    return QNN_OK;
}

qnn_status qnn_act_range(int kind, float s_out, int32_t z_out, int32_t *act_min, int32_t *act_max)
{
    if (act_min == nullptr || act_max == nullptr || kind < 0 || kind > 2) return QNN_EINVAL;
    if (!(s_out > 0.0f) || z_out < 0 || z_out > 255) return QNN_EINVAL;
    int32_t lo = (kind == 0) ? 0 : z_out;
    int32_t hi = 255;
    if (kind == 2) {
        const double six = std::fmin(qnn::nearest_away(6.0 / static_cast<double>(s_out)), 1.0e6);
        const long long top = static_cast<long long>(z_out) + static_cast<long long>(six);
        hi = static_cast<int32_t>(top > 255 ? 255 : top);
        if (hi < lo) hi = lo;
    }
    *act_min = lo;
    *act_max = hi;
    return QNN_OK;
}

qnn_status qnn_qadd_params(double s_a, double s_b, double s_out, int32_t *left_shift, int32_t *mult_a,
                           int32_t *shift_a, int32_t *mult_b, int32_t *shift_b, int32_t *mult_o, int32_t *shift_o)
{
    if (!left_shift || !mult_a || !shift_a || !mult_b || !shift_b || !mult_o || !shift_o) return QNN_EINVAL;
    if (!(s_a > 0.0) || !(s_b > 0.0) || !(s_out > 0.0)) return QNN_EINVAL;
    constexpr int kHeadroomBits = 20;
    const double common = 2.0 * std::fmax(s_a, s_b); // both inputs end up at most half of full scale
    *left_shift = kHeadroomBits;
    qnn_status st = qnn_quantize_multiplier(s_a / common, mult_a, shift_a);
    if (st == QNN_OK) st = qnn_quantize_multiplier(s_b / common, mult_b, shift_b);
    if (st == QNN_OK) st = qnn_quantize_multiplier(common / (std::ldexp(1.0, kHeadroomBits) * s_out), mult_o, shift_o);
    return st;
}

// Sec. 2.2 eq. 7-11 (symmetric, z = 0) with one scale per output-channel kernel (Sec. 2.6).
qnn_status qnn_quantize_weights(const float *w, size_t channels, size_t per_channel, int bits, int restricted,
                                int8_t *wq, float *delta)
{
    if (!w || !wq || !delta || (bits != 8 && bits != 4) || channels == 0 || per_channel == 0) return QNN_EINVAL;
    const int top = (1 << (bits - 1)) - 1;
    const int bottom = restricted ? -top : -top - 1;
    for (size_t c = 0; c < channels; ++c) {
        const float *row = w + c * per_channel;
        double peak = 0.0;
        for (size_t i = 0; i < per_channel; ++i) peak = std::fmax(peak, std::fabs(static_cast<double>(row[i])));
        const float step = peak > 0.0 ? static_cast<float>(peak / top) : 1.0f;
        delta[c] = step;
        for (size_t i = 0; i < per_channel; ++i) {
            double v = qnn::nearest_away(static_cast<double>(row[i]) / static_cast<double>(step));
            v = std::fmin(std::fmax(v, static_cast<double>(bottom)), static_cast<double>(top));
            wq[c * per_channel + i] = static_cast<int8_t>(v);
        }
    }
    return QNN_OK;
}

qnn_status qnn_pack_int4(const int8_t *v, size_t n, uint8_t *packed)
{
    if (!v || !packed || (n % 2) != 0) return QNN_EINVAL;
    for (size_t i = 0; i < n; ++i)
        if (v[i] < -8 || v[i] > 7) return QNN_EINVAL;
    for (size_t j = 0; j < n; j += 2)
        packed[j / 2] = static_cast<uint8_t>((static_cast<uint8_t>(v[j]) & 0x0F) | (static_cast<uint8_t>(v[j + 1]) << 4));
    return QNN_OK;
}

} // extern "C"
