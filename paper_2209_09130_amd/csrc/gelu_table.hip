// Threshold table of the FFN1 epilogue (host code, built once per layer at create time).
//
// The epilogue's decision is a function of ONE binary32 number: with y = fmaf(float(acc), m[n], bias[n]),
//     code = Q(y) = clamp(rne(fl32(fl32(GELU64(y)) * inv_s)), -127, 127),      GELU64(y) = y/2 (1 + erf(y / sqrt 2)) in binary64.
// Q is a step function of y with at most a few hundred steps, monotone on either side of GELU's minimum
// (y* = -0.7518): non-decreasing above it, non-increasing below it (every operation in it is monotone).
// So instead of evaluating GELU per element, the kernel looks the answer up: the y axis is cut into
// uniform bins narrow enough that Q changes at most once inside a bin, and bin i stores the binary32
// number Y_i at which it changes together with the codes on either side,
//     code = y >= Y_i ? hi_i : lo_i.
// The thresholds are found by bisection over the binary32 numbers with the definition above, so the
// lookup returns exactly what the definition returns, for every y, with no approximation left to certify.
// The bin of y comes out of one fused multiply-add whose addend carries 2^23: the sum is rounded to an
// integer by the adder and the integer sits in the low mantissa bits; the builder below evaluates the
// same expression to find each bin's first and last number, so that both sides agree on the bins.
#include "samp_common.h"

#include <cmath>
#include <cstring>

namespace samp {
namespace {

constexpr float TWO23 = 8388608.0f;
constexpr double GELU_ARGMIN = -0.75179;           // GELU decreases below it and increases above it

int q_exact(float y, float inv_s)
{
    const double yd = (double)y;
    const double g = 0.5 * yd * (1.0 + std::erf(yd * 0.70710678118654752440));
    const float v = (float)g * inv_s;
    float r = std::nearbyintf(v);                  // round half to even (default rounding mode)
    r = std::fmin(std::fmax(r, -127.0f), 127.0f);
    return (int)r;
}

double gelu_scaled(double y, double inv_s) { return 0.5 * y * (1.0 + std::erf(y * 0.70710678118654752440)) * inv_s; }

// binary32 numbers in their numeric order: key(a) < key(b)  <=>  a < b  (finite numbers, -0 just below +0)
int32_t key_of(float f)
{
    int32_t b;
    std::memcpy(&b, &f, 4);
    return b >= 0 ? b : (int32_t)(0x80000000u - (uint32_t)b) - 1;
}
float float_of(int32_t k)
{
    const int32_t b = k >= 0 ? k : (int32_t)(0x80000000u - (uint32_t)(k + 1));
    float f;
    std::memcpy(&f, &b, 4);
    return f;
}

int bin_of(float y, const GeluTableSpec &sp)
{
    float t = std::fmaf(y, sp.rate, sp.offset);
    t = std::fmin(std::fmax(t, TWO23), sp.t_max);
    uint32_t b;
    std::memcpy(&b, &t, 4);
    return (int)(b - 0x4B000000u);
}

// smallest binary32 number whose bin is >= i (i >= 1)
float first_of_bin(int i, const GeluTableSpec &sp)
{
    int64_t lo = key_of(-3.0e38f), hi = key_of(3.0e38f);          // bin(lo) = 0 < i <= bin(hi)
    while (hi - lo > 1) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (bin_of(float_of((int32_t)mid), sp) >= i) hi = mid; else lo = mid;
    }
    return float_of((int32_t)hi);
}

// Q is monotone on [a, b] and Q(a) != Q(b): smallest number in (a, b] at which Q already equals Q(b)
float change_point(float a, float b, float inv_s)
{
    const int qb = q_exact(b, inv_s);
    int64_t lo = key_of(a), hi = key_of(b);
    while (hi - lo > 1) {
        const int64_t mid = lo + (hi - lo) / 2;
        if (q_exact(float_of((int32_t)mid), inv_s) == qb) hi = mid; else lo = mid;
    }
    return float_of((int32_t)hi);
}

}  // namespace

bool gelu_table_plan(float inv_s, int refine, GeluTableSpec *sp)
{
    if (!(inv_s > 0.0f) || !std::isfinite(inv_s)) return false;
    const double k = (double)inv_s;
    // above y_hi the code is 127, below y_lo it is 0: the two ends of the table
    if (!(gelu_scaled(1.0e4, k) >= 128.0)) return false;
    double a = 0.0, b = 1.0e4;
    for (int it = 0; it < 200; it++) { const double m = 0.5 * (a + b); if (gelu_scaled(m, k) >= 128.0) b = m; else a = m; }
    const double y_hi = b;
    if (!(std::fabs(gelu_scaled(-38.0, k)) < 0.25)) return false;
    double y_lo = -0.76;
    if (!(std::fabs(gelu_scaled(y_lo, k)) < 0.25)) {
        a = -38.0; b = -0.76;                                       // |GELU| grows from a to b
        for (int it = 0; it < 200; it++) { const double m = 0.5 * (a + b); if (std::fabs(gelu_scaled(m, k)) < 0.25) a = m; else b = m; }
        y_lo = a;
    }
    // GELU's slope is at most 1.13, so consecutive steps of Q are at least (1/inv_s) / 1.13 apart
    double width = 0.6 / (1.13 * k);
    for (int r = 0; r < refine; r++) width /= 1.5;
    const double rate = 1.0 / width;
    const double bins = std::ceil((y_hi - y_lo) * rate) + 3.0;
    if (!(bins <= (double)GELU_TABLE_MAX_BINS)) return false;
    sp->rate = (float)rate;
    sp->offset = (float)((double)TWO23 + 1.0 - y_lo * rate);
    sp->bins = (int)bins;
    sp->t_max = TWO23 + (float)(sp->bins - 1);
    return sp->rate > 0.0f && std::isfinite(sp->rate) && std::isfinite(sp->offset);
}

bool gelu_table_fill(float inv_s, const GeluTableSpec &sp, uint32_t *entries)
{
    const float ystar = (float)GELU_ARGMIN;
    float first = -3.0e38f;
    for (int i = 0; i < sp.bins; i++) {
        const float next = i + 1 < sp.bins ? first_of_bin(i + 1, sp) : 3.0e38f;
        const float last = i + 1 < sp.bins ? float_of(key_of(next) - 1) : 3.0e38f;
        if (bin_of(first, sp) != i || bin_of(last, sp) != i) return false;          // an empty bin: the map is too fine
        const int q_first = q_exact(first, inv_s), q_last = q_exact(last, inv_s);
        float y_change = INFINITY;
        int lo = q_first, hi = q_first;
        if (first < ystar && ystar < last) {
            // the bin that holds the minimum: monotone on either half, at most one half may hold a step
            const int q_mid = q_exact(ystar, inv_s);
            const bool left = q_mid != q_first, right = q_mid != q_last;
            if (left && right) return false;
            if (left) { if (std::abs(q_mid - q_first) != 1) return false; y_change = change_point(first, ystar, inv_s); hi = q_mid; }
            if (right) { if (std::abs(q_last - q_mid) != 1) return false; y_change = change_point(ystar, last, inv_s); hi = q_last; }
        } else if (q_first != q_last) {
            if (std::abs(q_last - q_first) != 1) return false;                       // two steps in one bin: too coarse
            y_change = change_point(first, last, inv_s);
            hi = q_last;
        }
        std::memcpy(&entries[2 * i], &y_change, 4);
        entries[2 * i + 1] = ((uint32_t)lo & 0xffu) | (((uint32_t)hi & 0xffu) << 8);
        first = next;
    }
    // the ends must be the saturated codes, so that numbers beyond the table are answered by its end bins
    return q_exact(-3.0e38f, inv_s) == (int)(int8_t)(entries[1] & 0xff) && q_exact(3.0e38f, inv_s) == 127 &&
           (int)(int8_t)((entries[2 * sp.bins - 1] >> 8) & 0xff) == 127;
}

bool gelu_table_build(float inv_s, GeluTableSpec *sp, uint32_t *entries)
{
    for (int refine = 0; refine < 4; refine++) {
        if (!gelu_table_plan(inv_s, refine, sp)) return false;
        if (gelu_table_fill(inv_s, *sp, entries)) return true;
    }
    return false;
}

}  // namespace samp
