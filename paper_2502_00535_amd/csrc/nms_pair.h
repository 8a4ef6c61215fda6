// The pair test of the map step (Algorithm 1 of the paper) as evaluated on gfx950,
// and the host-side derivation of the per-threshold constants it needs.
//
// Definition to reproduce bit for bit (float32, round-to-nearest-even, one rounding
// per operation):
//     iw = max(0, (min(x2_v, x2_c) - max(x1_v, x1_c)) + 1)
//     ih = max(0, (min(y2_v, y2_c) - max(y1_v, y1_c)) + 1)
//     eliminated  <=>  not( (iw * ih) / area_c  <  theta )
// v = victim (lower rank), c = the outranking box, area_c = ((x2_c-x1_c)+1)*((y2_c-y1_c)+1).
//
// A correctly rounded float32 division costs about ten VALU instructions on CDNA.
// The fast form below reaches the same decision with one FMA and one compare:
//
//     q = RN(inter / area) >= theta
//       <=>  inter / area  >=  m          (m = theta - h, the rounding boundary just below
//                                          theta; h = half the gap to theta's predecessor)
//       <=>  inter - theta*area  >=  -h*area
//
// (inter / area == m exactly cannot happen, so the tie rule of the rounding never
// matters: in units of h, m is an odd integer of 25 bits, so m*area has an odd part
// of more than 24 bits and is not a float32, whereas inter is one.)
//
// E = inter - theta*area is what fma(-theta, area, inter) computes with a single
// rounding.  theta*area is a multiple of 2^(e_theta+e_area-46).  Whenever
// |E| < 2^(e_theta+e_area-22), inter is at least 2^(e_theta+e_area-1), so its own ulp
// is a multiple of that same unit, hence E is an integer below 2^24 times that unit
// and the FMA returns E exactly.  Otherwise the rounded value keeps E's sign and
// stays at or beyond 2^(e_theta+e_area-22) in magnitude, which exceeds h*area
// (< 2^(e_theta+e_area-23)).  Either way comparing the FMA result with -h*area
// (exact: h is a power of two) decides exactly as the division does.
//
// Two further savings, valid because the fast form is only used for theta > 0:
// the floor at zero is applied to one extent only (if the other is negative the
// product is <= 0 and the test fails, exactly as it does for a product floored to 0).
//
// The fast form is used for 2^-40 <= theta <= 2^20 (no overflow or underflow can
// occur for areas in [1, 2^82]); any other theta takes the literal division form.
#pragma once

#include <math.h>
#include <stdint.h>
#include <string.h>

#if defined(__HIPCC__)
#define NMS_HD __host__ __device__ __forceinline__
#else
#define NMS_HD static inline
#endif

struct NmsThetaConst {
    float theta;      // threshold as given
    float neg_theta;  // -theta
    float neg_h;      // -(half the distance from theta down to the next float32)
    int fast;         // 1: the FMA form is valid for this theta
};

static inline NmsThetaConst nms_make_theta_const(float theta)
{
    NmsThetaConst k;
    k.theta = theta;
    k.neg_theta = -theta;
    k.neg_h = 0.0f;
    k.fast = 0;
    if (theta >= 0x1p-40f && theta <= 0x1p20f) {
        uint32_t bits;
        memcpy(&bits, &theta, sizeof bits);
        uint32_t below = bits - 1u;  // predecessor of a positive normal float
        float pred;
        memcpy(&pred, &below, sizeof pred);
        float gap = theta - pred;  // exact (neighbouring floats)
        k.neg_h = -0.5f * gap;     // exact (power of two)
        k.fast = 1;
    }
    return k;
}

// Literal form: the definition, operation by operation.
NMS_HD bool nms_eliminates_exact(float vx1, float vy1, float vx2, float vy2,
                                 float cx1, float cy1, float cx2, float cy2,
                                 float c_area, float theta)
{
    float iw = fmaxf(0.0f, (fminf(vx2, cx2) - fmaxf(vx1, cx1)) + 1.0f);
    float ih = fmaxf(0.0f, (fminf(vy2, cy2) - fmaxf(vy1, cy1)) + 1.0f);
    float q = (iw * ih) / c_area;
    return !(q < theta);
}

// Fast form.  c_ng = neg_h * c_area (per outranking box, exact).
NMS_HD bool nms_eliminates_fast(float vx1, float vy1, float vx2, float vy2,
                                float cx1, float cy1, float cx2, float cy2,
                                float c_area, float c_ng, float neg_theta)
{
    float iw = (fminf(vx2, cx2) - fmaxf(vx1, cx1)) + 1.0f;  // may be negative, see above
    float ih = fmaxf(0.0f, (fminf(vy2, cy2) - fmaxf(vy1, cy1)) + 1.0f);
    float inter = iw * ih;
    float e = fmaf(neg_theta, c_area, inter);
    return e >= c_ng;
}

// Area of a box, pixel-inclusive (Algorithm 1's first assignment, one extent per axis).
NMS_HD float nms_box_area(float x1, float y1, float x2, float y2)
{
    return ((x2 - x1) + 1.0f) * ((y2 - y1) + 1.0f);
}
