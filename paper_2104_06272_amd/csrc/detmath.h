// Elementary functions as fixed sequences of correctly rounded binary32
// operations (add, mul, fma, div, sqrt), so that sampled actions and the
// pendulum's transitions come out bit-identical wherever they are evaluated.
// Compile with contraction off; every fused multiply-add below is explicit.
#pragma once
#include <math.h>
#include "philox.h"

namespace ank {

ANK_HD float f_from_bits(uint32_t u)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __uint_as_float(u);
#else
    float f; __builtin_memcpy(&f, &u, 4); return f;
#endif
}
ANK_HD uint32_t bits_from_f(float f)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __float_as_uint(f);
#else
    uint32_t u; __builtin_memcpy(&u, &f, 4); return u;
#endif
}

// e^x, argument clamped to [-87, 88] so the 2^n scaling stays a normal number
ANK_HD float det_exp(float x)
{
    x = x < -87.0f ? -87.0f : x;
    x = x > 88.0f ? 88.0f : x;
    const float n = rintf(x * 0x1.715476p+0f);
    float f = fmaf(-n, 0x1.62ep-1f, x);
    f = fmaf(-n, 0x1.0bfbe8p-15f, f);
    float p = 0x1.a01a02p-13f;
    p = fmaf(p, f, 0x1.6c16c2p-10f);
    p = fmaf(p, f, 0x1.111112p-7f);
    p = fmaf(p, f, 0x1.555556p-5f);
    p = fmaf(p, f, 0x1.555556p-3f);
    p = fmaf(p, f, 0.5f);
    p = fmaf(p, f, 1.0f);
    p = fmaf(p, f, 1.0f);
    const int e = (int)n + 127;
    return p * f_from_bits((uint32_t)e << 23);
}

// ln x for positive normal x
ANK_HD float det_log(float x)
{
    const uint32_t u = bits_from_f(x);
    int e = (int)(u >> 23) - 127;
    float m = f_from_bits((u & 0x007fffffu) | 0x3f800000u);
    if (m > 0x1.6a09e6p+0f) { m = m * 0.5f; e += 1; }
    const float s = (m - 1.0f) / (m + 1.0f);
    const float s2 = s * s;
    float p = 0x1.745d18p-4f;
    p = fmaf(p, s2, 0x1.c71c72p-4f);
    p = fmaf(p, s2, 0x1.24924ap-3f);
    p = fmaf(p, s2, 0x1.99999ap-3f);
    p = fmaf(p, s2, 0x1.555556p-2f);
    p = fmaf(p, s2, 1.0f);
    const float lm = (s + s) * p;
    const float fe = (float)e;
    const float r = fmaf(fe, 0x1.0bfbe8p-15f, lm);
    return fmaf(fe, 0x1.62ep-1f, r);
}

ANK_HD float det_sin_poly(float r)
{
    const float r2 = r * r;
    float p = 0x1.71de3ap-19f;
    p = fmaf(p, r2, -0x1.a01a02p-13f);
    p = fmaf(p, r2, 0x1.111112p-7f);
    p = fmaf(p, r2, -0x1.555556p-3f);
    p = p * r2;
    return fmaf(p, r, r);
}
ANK_HD float det_cos_poly(float r)
{
    const float r2 = r * r;
    float p = -0x1.27e4fcp-22f;
    p = fmaf(p, r2, 0x1.a01a02p-16f);
    p = fmaf(p, r2, -0x1.6c16c2p-10f);
    p = fmaf(p, r2, 0x1.555556p-5f);
    p = fmaf(p, r2, -0.5f);
    return fmaf(p, r2, 1.0f);
}

// sin and cos of an angle in [-pi_f, pi_f]
ANK_HD void det_sincos(float th, float& s, float& c)
{
    const float q = rintf(th * 0x1.45f306p-1f);
    float r = fmaf(-q, 0x1.92p+0f, th);
    r = fmaf(-q, 0x1.fb5444p-12f, r);
    const float sp = det_sin_poly(r), cp = det_cos_poly(r);
    const int qi = (int)q & 3;
    if (qi == 0)      { s = sp;  c = cp;  }
    else if (qi == 1) { s = cp;  c = -sp; }
    else if (qi == 2) { s = -sp; c = -cp; }
    else              { s = -cp; c = sp;  }
}

// cos(2 pi u), u in [0,1)
ANK_HD float det_cos2pi(float u)
{
    const float q = rintf(4.0f * u);
    const float r = fmaf(-0.25f, q, u);
    const float a = 0x1.921fb6p+2f * r;
    const int qi = (int)q & 3;
    if (qi == 0) return det_cos_poly(a);
    if (qi == 1) return -det_sin_poly(a);
    if (qi == 2) return -det_cos_poly(a);
    return det_sin_poly(a);
}

ANK_HD float det_tanh(float z)
{
    const float a = fabsf(z);
    float t;
    if (a < 0.25f) {
        const float a2 = a * a;
        float p = -0x1.226e36p-7f;
        p = fmaf(p, a2, 0x1.664f48p-6f);
        p = fmaf(p, a2, -0x1.ba1ba2p-5f);
        p = fmaf(p, a2, 0x1.111112p-3f);
        p = fmaf(p, a2, -0x1.555556p-2f);
        p = p * a2;
        t = fmaf(p, a, a);
    } else if (a > 9.0f) {
        t = 1.0f;
    } else {
        const float e = det_exp(-2.0f * a);
        t = (1.0f - e) / (1.0f + e);
    }
    return copysignf(t, z);
}

// bfloat16 bits of a finite binary32 value, round to nearest even
ANK_HD uint16_t bf16_bits(float x)
{
    uint32_t u = bits_from_f(x);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
ANK_HD float bf16_to_f(uint16_t h) { return f_from_bits((uint32_t)h << 16); }

}  // namespace ank
