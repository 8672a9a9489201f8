// The two 2048-entry twiddle tables as compile-time constants.
//
//   hi[h] = exp(-2 pi i h / 2^11),   lo[l] = exp(-2 pi i l / 2^22)
//
// They live in the code object's data segment, so a process gets them with the library itself: no allocation,
// no copy and no fill kernel on any stream, and the first call of the library may sit inside a stream capture.
// Values: the angle is reduced to the first octant in integer arithmetic (so 0, +-1 and +-sqrt(1/2) come out
// exactly where they belong), sine and cosine of the reduced angle are Taylor sums in double (remainder below
// 1e-19 for |x| <= pi/4), and the result is rounded once to binary32.
#pragma once
#include <stdint.h>

namespace fftsp {
namespace twtab {

struct Pair {
    float x, y;
};
struct alignas(256) Table {
    Pair v[2048];
};

constexpr double kTwoPi = 6.283185307179586476925286766559;

constexpr double sin_octant(double x)  // |x| <= pi/4
{
    const double x2 = x * x;
    double term = x, sum = x;
    for (int k = 1; k <= 10; ++k) {
        term *= -x2 / (double)((2 * k) * (2 * k + 1));
        sum += term;
    }
    return sum;
}
constexpr double cos_octant(double x)  // |x| <= pi/4
{
    const double x2 = x * x;
    double term = 1.0, sum = 1.0;
    for (int k = 1; k <= 10; ++k) {
        term *= -x2 / (double)((2 * k - 1) * (2 * k));
        sum += term;
    }
    return sum;
}

// exp(-2 pi i idx / 2^LOGN)
template <int LOGN>
constexpr Pair root(uint32_t idx)
{
    static_assert(LOGN >= 3, "octant reduction needs at least eight roots");
    constexpr uint32_t N = 1u << LOGN, Q = N / 8;
    const uint32_t i = idx & (N - 1u), oct = i / Q, r = i % Q;
    // alpha = angle past the octant's start, beta = angle up to the octant's end
    const double alpha = kTwoPi * (double)r / (double)N, beta = kTwoPi * (double)(Q - r) / (double)N;
    const double sa = sin_octant(alpha), ca = cos_octant(alpha), sb = sin_octant(beta), cb = cos_octant(beta);
    double c = 0, s = 0;
    switch (oct) {
        case 0: c = ca; s = sa; break;
        case 1: c = sb; s = cb; break;
        case 2: c = -sa; s = ca; break;
        case 3: c = -cb; s = sb; break;
        case 4: c = -ca; s = -sa; break;
        case 5: c = -sb; s = -cb; break;
        case 6: c = sa; s = -ca; break;
        default: c = cb; s = -sb; break;
    }
    return Pair{(float)c, (float)-s};
}

template <int LOGN>
constexpr Table make_table()
{
    Table t{};
    for (uint32_t i = 0; i < 2048u; ++i) t.v[i] = root<LOGN>(i);
    return t;
}

}  // namespace twtab
}  // namespace fftsp
