// Roots of unity and bf16 rounding evaluated by the compiler, for constant MFMA operand tables.
#pragma once

#include <stdint.h>

namespace monarch {
namespace croots {

// cos / sin of 2*pi*e/N for integer e, exact octant handling plus a Taylor series on [0, pi/4].
constexpr double kTwoPi = 6.283185307179586476925286766559;
constexpr double taylor_sin(double x) { double t = x, s = x; for (int k = 1; k < 12; ++k) { t *= -x * x / ((2 * k) * (2 * k + 1)); s += t; } return s; }
constexpr double taylor_cos(double x) { double t = 1, s = 1; for (int k = 1; k < 12; ++k) { t *= -x * x / ((2 * k - 1) * (2 * k)); s += t; } return s; }
struct CosSin { double c, s; };
constexpr CosSin unit_root(int e, int N)   // exp(+2 pi i e / N), N divisible by 8
{
    e %= N;
    const int quadrant = e / (N / 4), r = e % (N / 4);
    // first quadrant: angle r, mirrored around N/8 so that the series argument is <= pi/4
    const bool mirror = r > N / 8;
    const double x = kTwoPi * (mirror ? N / 4 - r : r) / N;
    const double c0 = mirror ? taylor_sin(x) : taylor_cos(x), s0 = mirror ? taylor_cos(x) : taylor_sin(x);
    switch (quadrant) {
    case 0: return {c0, s0};
    case 1: return {-s0, c0};
    case 2: return {-c0, -s0};
    default: return {s0, -c0};
    }
}
constexpr uint32_t bf16_bits(double v)     // round to nearest even
{
    const uint32_t x = __builtin_bit_cast(uint32_t, (float)v);
    return (x + 0x7fffu + ((x >> 16) & 1u)) >> 16;
}

}  // namespace croots
}  // namespace monarch
