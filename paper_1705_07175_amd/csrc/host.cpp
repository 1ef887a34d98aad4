// Host-side entry points of the binary-network library: status strings and the
// load-time fold of batch-norm + sign (Sec. 5.2 batch-norm layer, Eq. 1 of
// arXiv 1705.07175) into one integer threshold per channel.
//
// Compiled with -ffp-contract=off: every operation of y(x) rounds to double.
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>

#include "espresso_hip.h"

namespace {

constexpr int64_t kRange = 1ll << 30; // thresholds are exact for every integer |x| <= 2^30

struct Channel {
    double g, b, m, s;
    // y(x) = gamma * (x - mean) / sqrt(var + eps) + beta, left to right.
    bool nonneg(int64_t x) const { return nonneg(static_cast<double>(x)); }
    bool nonneg(double x) const
    {
        const double d = x - m;
        const double t = g * d;
        const double q = t / s;
        const double y = q + b;
        return y >= 0.0;
    }
};

// Smallest x in [lo, hi] at which pred flips from `first` to !first, for a predicate that
// is `first` on a (possibly empty) prefix and !first on the rest; hi + 1 if it never flips.
template <class Pred>
int64_t first_change(int64_t lo, int64_t hi, bool first, Pred pred)
{
    if (pred(lo) != first)
        return lo;
    if (pred(hi) == first)
        return hi + 1;
    // invariant: pred(lo) == first, pred(hi) != first
    while (hi - lo > 1) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (pred(mid) == first)
            lo = mid;
        else
            hi = mid;
    }
    return hi;
}

// Finite floats in increasing order <-> consecutive unsigned keys.
uint32_t float_key(float f)
{
    uint32_t u;
    std::memcpy(&u, &f, 4);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

float key_float(uint32_t k)
{
    const uint32_t u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    float f;
    std::memcpy(&f, &u, 4);
    return f;
}

} // namespace

extern "C" const char *esp_strerror(int status)
{
    switch (status) {
    case ESP_OK: return "ESP_OK";
    case ESP_EINVAL: return "ESP_EINVAL: null pointer or non-positive dimension";
    case ESP_EALIGN: return "ESP_EALIGN: buffer not aligned for its element type";
    case ESP_ESHAPE: return "ESP_ESHAPE: inconsistent or unsupported shape";
    case ESP_EWORKSPACE: return "ESP_EWORKSPACE: workspace missing or too small";
    case ESP_ELAUNCH: return "ESP_ELAUNCH: the HIP runtime refused a kernel launch";
    default: return "unknown esp_status";
    }
}

extern "C" int esp_version(void) { return 100; }

extern "C" int esp_bn_fold(const float *gamma, const float *beta, const float *mean, const float *var,
                           float eps, int C, int32_t *thr, uint64_t *flip)
{
    if (C <= 0 || !gamma || !beta || !mean || !var || !thr || !flip)
        return ESP_EINVAL;
    const int Cw = (C + 63) / 64;
    for (int w = 0; w < Cw; ++w)
        flip[w] = 0;
    constexpr int32_t kAlways = std::numeric_limits<int32_t>::min(); // x >= kAlways for every x

    for (int c = 0; c < C; ++c) {
        Channel ch;
        ch.g = static_cast<double>(gamma[c]);
        ch.b = static_cast<double>(beta[c]);
        ch.m = static_cast<double>(mean[c]);
        ch.s = std::sqrt(static_cast<double>(var[c]) + static_cast<double>(eps));
        auto pred = [&](int64_t x) { return ch.nonneg(x); };

        bool flipped = false;
        int32_t t = kAlways;
        if (ch.g > 0.0) {
            // y is non-decreasing in x (every rounding step is monotone): bit = (x >= thr)
            const int64_t x0 = first_change(-kRange, kRange, false, pred);
            if (x0 > kRange) {        // never non-negative in range: constant 0
                t = kAlways;
                flipped = true;
            } else if (x0 <= -kRange) // always non-negative: constant 1
                t = kAlways;
            else
                t = static_cast<int32_t>(x0);
        } else if (ch.g < 0.0) {
            // y is non-increasing: non-negative up to some x*, then negative: bit = !(x >= x*+1)
            const int64_t x0 = first_change(-kRange, kRange, true, pred);
            flipped = true;
            if (x0 > kRange) {        // non-negative over the whole range: constant 1
                t = kAlways;
                flipped = false;
            } else if (x0 <= -kRange) // negative over the whole range: constant 0
                t = kAlways;
            else
                t = static_cast<int32_t>(x0);
        } else {
            // gamma == 0 (or NaN): y does not depend on x over the legal range
            flipped = !pred(0);
            t = kAlways;
        }
        thr[c] = t;
        if (flipped)
            flip[c / 64] |= 1ull << (c % 64);
    }
    return ESP_OK;
}

extern "C" int esp_bn_fold_f32(const float *gamma, const float *beta, const float *mean, const float *var,
                               float eps, int C, float *thr, float *sgn)
{
    if (C <= 0 || !gamma || !beta || !mean || !var || !thr || !sgn)
        return ESP_EINVAL;
    const float inf = std::numeric_limits<float>::infinity();
    const int64_t lo = float_key(-std::numeric_limits<float>::max());
    const int64_t hi = float_key(std::numeric_limits<float>::max());
    for (int c = 0; c < C; ++c) {
        Channel ch;
        ch.g = static_cast<double>(gamma[c]);
        ch.b = static_cast<double>(beta[c]);
        ch.m = static_cast<double>(mean[c]);
        ch.s = std::sqrt(static_cast<double>(var[c]) + static_cast<double>(eps));
        auto pred = [&](int64_t k) {
            return ch.nonneg(static_cast<double>(key_float(static_cast<uint32_t>(k))));
        };
        float t = -inf, sg = 1.0f; // default: constant 1 (every finite x >= -inf)
        if (ch.g > 0.0) {
            const int64_t k0 = first_change(lo, hi, false, pred);
            if (k0 > hi)
                t = inf;            // never non-negative: constant 0
            else if (k0 > lo)
                t = key_float(static_cast<uint32_t>(k0));
        } else if (ch.g < 0.0) {
            const int64_t k0 = first_change(lo, hi, true, pred); // first x with y(x) < 0
            if (k0 <= lo)
                t = inf;            // negative everywhere: constant 0
            else if (k0 <= hi) {    // y >= 0 iff x <= x* = float(k0 - 1) iff -x >= -x*
                t = -key_float(static_cast<uint32_t>(k0 - 1));
                sg = -1.0f;
            }
        } else if (!pred(float_key(0.0f))) {
            t = inf;                // gamma == 0 (or NaN): constant sign of beta
        }
        thr[c] = t;
        sgn[c] = sg;
    }
    return ESP_OK;
}
