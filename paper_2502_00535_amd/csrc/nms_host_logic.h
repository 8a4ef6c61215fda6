// Index arithmetic, sort keys and workspace layout of the NMS library: plain functions with no
// device-only construct in them, shared by the kernels and the launch code and compilable by a
// host compiler alone (the host tests sweep them without a GPU).
#pragma once

#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#include "nms_pair.h"  // NMS_HD

// ---- rank keys ----------------------------------------------------------------------------
// Unique ascending 64-bit key of (score, index): a better score sorts first, equal scores by
// lower index; -0.0 ties with +0.0.  Valid for every float but NaN (negative scores, denormals
// and both infinities order as the numbers they are).
NMS_HD unsigned long long nms_rank_key(float score, unsigned idx)
{
    unsigned u;
    memcpy(&u, &score, sizeof u);
    if (u == 0x80000000u) u = 0u;
    const unsigned asc = (u & 0x80000000u) ? ~u : (u | 0x80000000u);  // ascending in the score
    return ((unsigned long long)(~asc) << 32) | idx;
}

// ---- work units of the map step -------------------------------------------------------------
// One unit = one column tile tc (64 outranking boxes) against a "super-row" of kSuper
// consecutive victim tile rows, i.e. up to kSuper tiles of the ranked lower triangle.
// Super-row sr has min(kSuper*(sr+1), T) units (tc = 0 .. last tile row of the super-row), so
// the units before super-row sr number kSuper * sr*(sr+1)/2.

// Number of units for T tile rows.
NMS_HD int nms_triangle_units(int T, int super)
{
    const int SR = (T + super - 1) / super;
    return SR == 0 ? 0 : super * (SR - 1) * SR / 2 + T;
}

// Linear unit index g -> (sr, tc): the largest sr with kSuper*sr*(sr+1)/2 <= g, by a float
// square root and a correction in exact integer arithmetic.
template <int kSuper>
NMS_HD void nms_triangle_unit(int g, int &sr, int &tc)
{
    int r = (int)((sqrtf(1.0f + (8.0f / kSuper) * (float)g) - 1.0f) * 0.5f);
    while ((long long)kSuper * r * (r + 1) / 2 > g) --r;
    while ((long long)kSuper * (r + 1) * (r + 2) / 2 <= g) ++r;
    sr = r;
    tc = g - kSuper * r * (r + 1) / 2;
}

// ---- workspace of the whole-path calls --------------------------------------------------------
NMS_HD size_t nms_align256(size_t v) { return (v + 255) & ~(size_t)255; }

// Byte offsets of the parts of the workspace (every part 256-byte aligned), for frames of at most
// n_max boxes, n_pad = n_max rounded up to a multiple of 64.  `end` is the size.
struct NmsRunLayout {
    size_t order;    // int32 [frames][n_max]          rank -> input index
    size_t sorted5;  // float [frames][5 * n_pad]      box table: rows (x1,y1,x2,y2), then areas
    size_t ysc;      // float4 [frames][n_pad]         boxes with y * 2^-14, rank order
    size_t ytile;    // uint32 [frames][n_pad / 64]    1 = every box of the tile may use the y-scaled form
    size_t tsc;      // float [frames][n_pad]          per box, 2^-14 x the float32 its intersections are compared with
    size_t keys;     // uint64 [frames][n_pad]         chunk-sorted keys, only when n_max > sort_chunk
    size_t end;
};

NMS_HD NmsRunLayout nms_run_layout(int n_max, int n_pad, int frames, int sort_chunk)
{
    NmsRunLayout l;
    size_t p = 0;
    l.order = p;
    p += nms_align256((size_t)frames * (size_t)n_max * sizeof(int32_t));
    l.sorted5 = p;
    p += nms_align256((size_t)frames * 5 * (size_t)n_pad * sizeof(float));
    l.ysc = p;
    p += nms_align256((size_t)frames * (size_t)n_pad * 4 * sizeof(float));
    l.ytile = p;
    p += nms_align256((size_t)frames * (size_t)(n_pad / 64) * sizeof(uint32_t));
    l.tsc = p;
    p += nms_align256((size_t)frames * (size_t)n_pad * sizeof(float));
    l.keys = p;
    if (n_max > sort_chunk) p += nms_align256((size_t)frames * (size_t)n_pad * sizeof(unsigned long long));
    l.end = p;
    return l;
}
