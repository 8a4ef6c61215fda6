// The pair test of the map step (Algorithm 1 of the paper) as evaluated on gfx950,
// and the host-side derivation of the per-threshold constants it needs.
//
// Definition to reproduce bit for bit (float32, round-to-nearest-even, one rounding
// per operation):
//     iw = max(0, (min(x2_v, x2_c) - max(x1_v, x1_c)) + 1)
//     ih = max(0, (min(y2_v, y2_c) - max(y1_v, y1_c)) + 1)
//     inter = iw * ih
//     eliminated  <=>  not( inter / area_c  <  theta )
// v = victim (lower rank), c = the outranking box, area_c = ((x2_c-x1_c)+1)*((y2_c-y1_c)+1).
//
// A correctly rounded float32 division costs about ten VALU instructions on CDNA.
// The fast form replaces the division AND the threshold compare by one compare against
// a per-box constant that is worked out once per 64 victims:
//
//     RN(inter / area) >= theta
//       <=>  inter / area >= m        m = theta - h is the rounding boundary just below theta
//                                     (h = half the gap to theta's float32 predecessor);
//                                     everything at or above m rounds to theta or higher
//       <=>  inter >= m * area        (real numbers; area > 0)
//       <=>  inter >= T(area)         T = the smallest float32 that is >= m * area,
//                                     because inter itself is a float32
//
// m has 25 significant bits and area 24, so m * area is exact in float64, and T is that
// product converted to float32 rounding upwards.  (inter / area == m exactly cannot
// happen -- in units of h, m is an odd 25-bit integer, so m * area is never a float32 --
// hence the ties-to-even rule of the division never comes into play.)
//
// One further saving, valid because the fast form is only used for theta > 0: the floor
// at zero is applied to one extent only.  If the other extent is negative the product is
// <= 0 < T and the test fails, exactly as it does for a product floored to 0.
//
// The fast form is used for 2^-40 <= theta <= 2^20 (no overflow or underflow for areas
// in [1, 2^100]); any other theta takes the literal division form.
//
// y-scaled variant of the fast form.  max(0, .) is a half-rate VALU instruction on gfx950,
// whereas an add with the clamp output modifier (result limited to [0, 1]) runs at full
// rate and is the same thing as long as the sum stays below 1.  So the y coordinates are
// carried multiplied by S = 2^-14 and the "+1" becomes "+S":
//     ih_S = clamp01((min(y2_v S, y2_c S) - max(y1_v S, y1_c S)) + S)  =  S * ih
// Multiplying by a power of two commutes with every rounding involved as long as nothing
// leaves the normal range, which holds when every y is 0 or 2^-60 <= |y| <= 8190 (then
// differences are 0 or >= 2^-83, extents are 0 or >= 2^-24, ih <= 16381 < 2^14).  The
// product iw * ih_S = S * inter is compared with S * T.  Boxes are grouped in tiles of 64;
// a tile whose boxes do not all meet the condition is simply processed in the unscaled form.
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
    float theta;   // threshold as given
    double m;      // rounding boundary just below theta (exact in float64)
    int fast;      // 1: the compare-against-T form is valid for this theta
};

static inline NmsThetaConst nms_make_theta_const(float theta)
{
    NmsThetaConst k;
    k.theta = theta;
    k.m = 0.0;
    k.fast = 0;
    if (theta >= 0x1p-40f && theta <= 0x1p20f) {
        uint32_t bits;
        memcpy(&bits, &theta, sizeof bits);
        uint32_t below = bits - 1u;  // predecessor of a positive normal float
        float pred;
        memcpy(&pred, &below, sizeof pred);
        k.m = 0.5 * ((double)theta + (double)pred);  // exact: 25 significant bits
        k.fast = 1;
    }
    return k;
}

// T(area): smallest float32 >= m * area.  The product is exact in float64; the
// conversion rounds to nearest and is bumped to the next float32 when it fell short.
NMS_HD float nms_pair_threshold(float area, double m)
{
    const double prod = m * (double)area;
    float t = (float)prod;
    if ((double)t < prod) {
        uint32_t b;
        memcpy(&b, &t, sizeof b);
        b += 1u;  // next float32 up (t is positive and finite)
        memcpy(&t, &b, sizeof t);
    }
    return t;
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

// Fast form.  c_T = nms_pair_threshold(area of the outranking box, m).
NMS_HD bool nms_eliminates_fast(float vx1, float vy1, float vx2, float vy2,
                                float cx1, float cy1, float cx2, float cy2, float c_T)
{
    float iw = (fminf(vx2, cx2) - fmaxf(vx1, cx1)) + 1.0f;  // may be negative, see above
    float ih = fmaxf(0.0f, (fminf(vy2, cy2) - fmaxf(vy1, cy1)) + 1.0f);
    return iw * ih >= c_T;
}

// ---- y-scaled fast form ---------------------------------------------------------------
#define NMS_YSCALE 0x1p-14f

// May this y coordinate take part in the scaled form?
NMS_HD bool nms_y_regular(float y)
{
    const float a = fabsf(y);
    return a == 0.0f || (a >= 0x1p-60f && a <= 8190.0f);
}

// vy1s.. are y coordinates times NMS_YSCALE, c_Ts = NMS_YSCALE * T, y_one = NMS_YSCALE.
// (y_one is a parameter so that device code can keep it in a vector register: with a
// scalar-register or literal operand the add would drop to half rate.)
NMS_HD bool nms_eliminates_fast_yscaled(float vx1, float vy1s, float vx2, float vy2s,
                                        float cx1, float cy1s, float cx2, float cy2s, float c_Ts, float y_one)
{
    float iw = (fminf(vx2, cx2) - fmaxf(vx1, cx1)) + 1.0f;
    float ihs = (fminf(vy2s, cy2s) - fmaxf(vy1s, cy1s)) + y_one;
    ihs = fminf(fmaxf(ihs, 0.0f), 1.0f);  // folds into the add as its clamp modifier
    return iw * ihs >= c_Ts;
}

// ---- fast form, scaled late ------------------------------------------------------------
// Where no y-scaled table exists (or a tile is outside its range) the half-rate floor can
// still be avoided: ih = (min - max) + 1 as defined, then ih * NMS_YSCALE with the clamp
// modifier (full rate) instead of max(0, ih).  Scaling by a power of two is exact, a negative
// extent clamps to 0 as the floor would make it, and the product is compared with
// NMS_YSCALE * T.  The clamp's upper end must not bite: ih never exceeds the outranking box's
// own extent (y2_c - y1_c) + 1 (every step of both is monotone), so it is enough that this
// extent is at most 2^14 -- a condition on the outranking box alone.  (An extent below 2^-112,
// whose scaled value would leave the normal range, gives a product far below any T either way.)
// Costs one full-rate instruction more than the y-scaled table form, one half-rate
// instruction less than the plain fast form.
NMS_HD bool nms_extent_fits_late_scaling(float cy1, float cy2)
{
    return (cy2 - cy1) + 1.0f <= 16384.0f;
}

// c_Ts = NMS_YSCALE * T, y_scale = NMS_YSCALE (a parameter for the same reason as y_one above).
NMS_HD bool nms_eliminates_fast_latescaled(float vx1, float vy1, float vx2, float vy2,
                                           float cx1, float cy1, float cx2, float cy2, float c_Ts, float y_scale)
{
    float iw = (fminf(vx2, cx2) - fmaxf(vx1, cx1)) + 1.0f;
    float ih = (fminf(vy2, cy2) - fmaxf(vy1, cy1)) + 1.0f;
    float ihs = fminf(fmaxf(ih * y_scale, 0.0f), 1.0f);  // folds into the multiply as its clamp modifier
    return iw * ihs >= c_Ts;
}

// Area of a box, pixel-inclusive (Algorithm 1's first assignment, one extent per axis).
NMS_HD float nms_box_area(float x1, float y1, float x2, float y2)
{
    return ((x2 - x1) + 1.0f) * ((y2 - y1) + 1.0f);
}
