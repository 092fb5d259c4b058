// Per-sample loss terms and head gradients shared by the fused update kernels.
#pragma once
#include "internal.h"
#include "detmath.h"

namespace ank {

// loss terms and head gradient of one categorical sample with three actions and one value (NH = 4); the
// operation order is head_grad's
__device__ __forceinline__ void catch_head_grad(const float4 hv4, int act, float A_, float G_, float beta, float cv, float inv_m,
                                                float (&d)[4], float& lp_term, float& v_term, float& e_term)
{
    const float hv[3] = {hv4.x, hv4.y, hv4.z};
    const float dv = G_ - hv4.w;
    v_term = cv * dv * dv;
    float mx = hv[0];
#pragma unroll
    for (int j = 1; j < 3; ++j) mx = fmaxf(mx, hv[j]);
    float e[3], Z = 0.0f;
#pragma unroll
    for (int j = 0; j < 3; ++j) { e[j] = det_exp(hv[j] - mx); Z += e[j]; }
    const float logZ = det_log(Z), invZ = 1.0f / Z;
    float H = 0.0f, lpa = 0.0f, p[3], lp[3];
#pragma unroll
    for (int j = 0; j < 3; ++j) {
        lp[j] = hv[j] - mx - logZ;
        p[j] = e[j] * invZ;
        H -= p[j] * lp[j];
        if (j == act) lpa = lp[j];
    }
#pragma unroll
    for (int j = 0; j < 3; ++j) d[j] = (-A_ * ((j == act ? 1.0f : 0.0f) - p[j]) + beta * p[j] * (lp[j] + H)) * inv_m;
    d[3] = -2.0f * cv * dv * inv_m;
    lp_term = -A_ * lpa;
    e_term = -beta * H;
}

}  // namespace ank
