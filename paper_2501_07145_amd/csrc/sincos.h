// Accurate single-precision sin/cos for the feature kernels (internal header).
#pragma once

#include <hip/hip_runtime.h>

namespace rfsf {
namespace {

// sin and cos of x to ~1e-7 absolute for |x| up to 1e5: two-term Cody-Waite reduction by
// pi/2 with fused multiply-adds, then degree-7 / degree-8 minimax polynomials on
// [-pi/4, pi/4] and a quadrant swap. The time difference cancels leading digits, so the
// fast hardware approximations are not accurate enough here.
__device__ __forceinline__ void sincos_reduced(float x, float &s, float &c)
{
    const float kf = rintf(x * 0.636619772367581343f);
    float r = fmaf(-kf, 1.57079637050628662109375f, x);
    r = fmaf(-kf, -4.37113900018624283e-8f, r);
    const float r2 = r * r;
    const float ps = fmaf(r2, fmaf(r2, -1.9515295891e-4f, 8.3321608736e-3f), -1.6666654611e-1f);
    const float S = fmaf(r * r2, ps, r);
    const float pc = fmaf(r2, fmaf(r2, 2.443315711809948e-5f, -1.388731625493765e-3f), 4.166664568298827e-2f);
    const float C = fmaf(r2 * r2, pc, fmaf(-0.5f, r2, 1.0f));
    const int q = (int)kf;
    const float ss = (q & 1) ? C : S;
    const float cc = (q & 1) ? S : C;
    // sin flips sign in quadrants 2, 3; cos in quadrants 1, 2.
    s = __uint_as_float(__float_as_uint(ss) ^ (((unsigned)q & 2u) << 30));
    c = __uint_as_float(__float_as_uint(cc) ^ ((((unsigned)q + 1u) & 2u) << 30));
}

}  // namespace
}  // namespace rfsf
