// RoPE angle arithmetic shared by the decode kernels.
#ifndef CF_ROPE_DEVICE_H
#define CF_ROPE_DEVICE_H

#include <hip/hip_runtime.h>

namespace cf {

// Frequency of RoPE pair i: base^(-2i/head_dim), from log2(base), in fp64.
__device__ __forceinline__ double rope_inv_freq(int i, int head_dim, double log2_base)
{
    return exp2(-(2.0 * (double)i / (double)head_dim) * log2_base);
}

// cos and sin of pos * inv_freq, angle and range reduction in fp64.
__device__ __forceinline__ void rope_cos_sin(int pos, double inv_freq, float &cos_out, float &sin_out)
{
    const double ang = (double)pos * inv_freq;
    const double k = rint(ang * 0.63661977236758134308);              // 2/pi
    double r = fma(-k, 1.57079632679489655800e+00, ang);              // pi/2, high part
    r = fma(-k, 6.12323399573676603587e-17, r);                       // pi/2, low part
    const double r2 = r * r;                                          // |r| <= pi/4: Taylor series
    double s = -1.0 / 1307674368000.0;
    s = fma(s, r2, 1.0 / 6227020800.0);
    s = fma(s, r2, -1.0 / 39916800.0);
    s = fma(s, r2, 1.0 / 362880.0);
    s = fma(s, r2, -1.0 / 5040.0);
    s = fma(s, r2, 1.0 / 120.0);
    s = fma(s, r2, -1.0 / 6.0);
    s = fma(s * r2, r, r);
    double c = 1.0 / 20922789888000.0;
    c = fma(c, r2, -1.0 / 87178291200.0);
    c = fma(c, r2, 1.0 / 479001600.0);
    c = fma(c, r2, -1.0 / 3628800.0);
    c = fma(c, r2, 1.0 / 40320.0);
    c = fma(c, r2, -1.0 / 720.0);
    c = fma(c, r2, 1.0 / 24.0);
    c = fma(c, r2, -0.5);
    c = fma(c, r2, 1.0);
    const int q = (int)((long long)k & 3);
    const double sv = (q == 0) ? s : (q == 1) ? c : (q == 2) ? -s : -c;
    const double cv = (q == 0) ? c : (q == 1) ? -s : (q == 2) ? -c : s;
    cos_out = (float)cv;
    sin_out = (float)sv;
}

}  // namespace cf
#endif
