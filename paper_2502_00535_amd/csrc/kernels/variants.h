// Part of nms_kernels.hip (included there, inside its anonymous namespace): map step with the selectable measure / compare / ties / offset / labels.
#pragma once

// ----------------------------------------------------------------------------- map with options

// Rank-ordered scores, class labels and areas under the chosen pixel offset (victims of a row
// are fetched with scalar loads, so the map kernel wants them contiguous in rank order like
// the box table).
__global__ void __launch_bounds__(256)
gather_ranked_kernel(const int32_t *__restrict__ order, const float *__restrict__ scores,
                     const int32_t *__restrict__ classes, const int32_t *__restrict__ counts,
                     const float *__restrict__ sorted5, float offset, int n_max, int n_pad,
                     float *__restrict__ ranked_score, int32_t *__restrict__ ranked_class,
                     float *__restrict__ ranked_area)
{
    const int f = blockIdx.y;
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_pad) return;
    const int n_f = frame_count(counts, f, n_max);
    const bool real = r < n_f;
    const int idx = real ? order[(size_t)f * n_max + r] : 0;
    ranked_score[(size_t)f * n_pad + r] = real ? scores[(size_t)f * n_max + idx] : -INFINITY;
    if (classes != nullptr) ranked_class[(size_t)f * n_pad + r] = real ? classes[(size_t)f * n_max + idx] : 0;
    // area under the chosen pixel offset (the box table's own area column is the offset-1 one)
    const float4 b = reinterpret_cast<const float4 *>(sorted5 + (size_t)f * 5 * n_pad)[r];
    ranked_area[(size_t)f * n_pad + r] = ((b.z - b.x) + offset) * ((b.w - b.y) + offset);
}

// The map step with the selectable measure / compare / tie / label / offset variants, one
// wavefront per 64x64 tile of the ranked lower triangle, mask layout as in map_tile_kernel.
// The denominator changes per pair under intersection-over-union, so there is no per-box
// threshold to precompute; the division and the compare are still decided without dividing:
//     RN(inter / d) >= theta  <=>  inter >= m * d     m = rounding boundary just below theta
//     RN(inter / d) >  theta  <=>  inter >= m' * d    m' = rounding boundary just above theta
// (d > 0; equality with m*d or m'*d cannot occur, by the same argument as in nms_pair.h).  m and m'
// have 25 significant bits and d 24, so the product is exact in float64 and the compare is
// done there.  Thresholds outside [2^-40, 2^20] take the literal float32 division (kExDivide).
// Rank order puts equal scores next to each other, so "ties ignored" is the extra test
// score_c > score_r on the pairs the triangle already holds.
// IOU: the measure.  MODE: how the threshold is decided (above).  AUX: the launch uses the
// rank-ordered scores and / or labels (ties ignored, labels given).
// Work units and their mapping to workgroups are those of map_tile_kernel: one column tile
// against kSuper victim tiles per wavefront, frames pinned to XCDs on batches.
// WRITE_MASK: store the tiles' words for a reduce step (the greedy sweep needs them).
// Otherwise the row reduction of the paper's rule is folded in as in map_tile_kernel: keep_out
// was preset to 1 by the rank step and every victim with an eliminator gets a 0.
template <bool IOU, int MODE, bool AUX, int kSuper, bool WRITE_MASK>
__global__ void __launch_bounds__(kMapWaves * 64)
map_tile_ex_kernel(const float *__restrict__ sorted5, const float *__restrict__ ranked_score,
                   const int32_t *__restrict__ ranked_class, const float *__restrict__ ranked_area,
                   const int32_t *__restrict__ counts, int n_max, int n_pad,
                   int tiles, int tile_blocks, int frames, int xcd_frames, float theta, double boundary,
                   float boundary_lo, float offset, int flags, unsigned long long *__restrict__ mask, const int32_t *__restrict__ order,
                   uint8_t *__restrict__ keep_out)
{
    const int lane = threadIdx.x & 63;
    int f, bx;
    if (xcd_frames) {  // frame f runs entirely on XCD f mod 8 (see map_tile_kernel)
        const int slot = blockIdx.x >> 3;
        f = (slot / tile_blocks) * 8 + (int)(blockIdx.x & 7);
        bx = slot % tile_blocks;
        if (f >= frames) return;
    } else {
        f = blockIdx.y;
        bx = blockIdx.x;
    }
    const int g = __builtin_amdgcn_readfirstlane(bx * kMapWaves + (int)(threadIdx.x >> 6));
    if (g >= tiles) return;
    const int n_f = frame_count(counts, f, n_max);
    int sr, tc;
    nms_triangle_unit<kSuper>(g, sr, tc);
    const int tiles_f = (n_f + kTile - 1) / kTile;
    int tr = kSuper * sr > tc ? kSuper * sr : tc;
    const int tr_end = kSuper * sr + kSuper < tiles_f ? kSuper * sr + kSuper : tiles_f;
    if (tr >= tr_end) return;

    const float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    const float4 *box4 = reinterpret_cast<const float4 *>(sorted_f);
    const float *score_f = ranked_score + (size_t)f * n_pad;
    const int32_t *class_f = ranked_class + (size_t)f * n_pad;  // unwritten (but allocated) when no labels were given
    const float *area_f = ranked_area + (size_t)f * n_pad;
    const bool ties_ignore = (flags & kExTiesIgnore) != 0;
    const bool labelled = (flags & kExClasses) != 0;

    const int c = tc * kTile + lane;
    const float4 cb = box4[c];
    const float c_area = area_f[c];
    float off = offset;  // in a vector register: an add with a scalar-register source issues at half rate
    asm volatile("" : "+v"(off));
    const float c_score = AUX ? score_f[c] : 0.0f;
    const int c_class = AUX ? class_f[c] : 0;
    const float c_T = (MODE == kExBoundary && !IOU) ? nms_pair_threshold(c_area, boundary) : 0.0f;
    // Intersection over union, boundary form: the exact decision, inter >= boundary * denom, is a
    // float64 compare behind two more float32 operations for the denominator.  Most pairs are
    // nowhere near the threshold, so two float32 tests go first that can only err towards "maybe":
    //   1. the union is never smaller than the outranking box's own area -- as float32 values,
    //      denom >= c_area * (1 - 2^-22): the sum of the areas is at least the larger one, the
    //      intersection at most the smaller one, two roundings -- so with
    //      c_T1 = the float32 at or below boundary * c_area * (1 - 2^-21), worked out once per lane,
    //      inter < c_T1 is a certain miss.  One compare, like the outranking-area measure.
    //   2. rows in which some lane passed: with boundary_lo <= boundary * (1 - 2^-22),
    //      RN(denom * boundary_lo) < boundary * denom for every denominator of at least 2^-40 (the
    //      product's rounding error is 2^-24 relative), so inter < RN(denom * boundary_lo) is a certain
    //      miss too.  The condition on the denominator is checked once per work unit on the lanes'
    //      areas; a unit that fails it skips this test.
    // Rows that still hold a "maybe" are decided exactly.
    constexpr bool kPretest = IOU && MODE == kExBoundary;
    const bool pretest = kPretest && __ballot(c_area < 0x1p-40f) == 0ull;
    float c_lo = boundary_lo;  // in a vector register, like `off`
    asm volatile("" : "+v"(c_lo));
    float c_T1 = 0.0f;
    if (kPretest) {
        const double t = boundary * (double)c_area * (1.0 - 0x1p-21);
        c_T1 = (float)t;
        if ((double)c_T1 > t) c_T1 = __uint_as_float(__float_as_uint(c_T1) - 1u);  // next float32 down (t > 0)
        if (!(c_T1 > 0.0f)) c_T1 = 0.0f;
    }

    // one tile; DIAG: the tile on the diagonal, where only better-ranked boxes of the tile eliminate
    auto tile = [&](auto on_diagonal) __attribute__((always_inline)) {
        constexpr bool DIAG = decltype(on_diagonal)::value;
        const float4 *__restrict__ vb = box4 + tr * kTile;  // wave-uniform addresses: scalar loads
        const float *__restrict__ vs = score_f + tr * kTile;
        const int32_t *__restrict__ vc = class_f + tr * kTile;
        const float *__restrict__ va = area_f + tr * kTile;
        unsigned w_lo = 0, w_hi = 0;
        unsigned lane_hit = 0;  // fused form: lane r = 1 when row r has an eliminator in this tile
        constexpr int kGroup = 8;
#pragma unroll 1
        for (int grp = 0; grp < kTile / kGroup; ++grp) {
            // a group's victims are fetched together, its words formed without a branch in between
            float4 v[kGroup];
            float v_score[kGroup];
            int v_class[kGroup];
            float v_area[kGroup];
#pragma unroll
            for (int k = 0; k < kGroup; ++k) {
                v[k] = vb[kGroup * grp + k];
                v_area[k] = IOU ? va[kGroup * grp + k] : 0.0f;
                v_score[k] = AUX ? vs[kGroup * grp + k] : 0.0f;
                v_class[k] = AUX ? vc[kGroup * grp + k] : 0;
            }
            unsigned long long words[kGroup];
            unsigned grp_bits = 0;  // wave-uniform: bit k = row kGroup*grp+k has an eliminator
#pragma unroll
            for (int k = 0; k < kGroup; ++k) {
                const int r = kGroup * grp + k;
                // with a positive threshold boundary one floor is enough: a negative width times a
                // floored height is <= 0 and can reach neither T nor boundary * (a positive union)
                float iw = (fminf(v[k].z, cb.z) - fmaxf(v[k].x, cb.x)) + off;
                if (MODE != kExBoundary) iw = fmaxf(0.0f, iw);
                const float ih = fmaxf(0.0f, (fminf(v[k].w, cb.w) - fmaxf(v[k].y, cb.y)) + off);
                const float inter = iw * ih;
                bool hit;
                if (MODE == kExBoundary && !IOU)
                    hit = inter >= c_T;  // the denominator is the lane's own area: one float32 threshold per box, as in nms_pair.h
                else if (MODE == kExBoundary)
                    hit = inter >= c_T1;  // certain miss below it (see above); decided further down otherwise
                else if (MODE == kExDivideGe)
                    hit = !(inter / (IOU ? (v_area[k] + c_area) - inter : c_area) < theta);
                else
                    hit = inter / (IOU ? (v_area[k] + c_area) - inter : c_area) > theta;
                unsigned long long word = __ballot(hit);
                if (DIAG) word &= (1ull << r) - 1ull;
                if (AUX && word != 0) {  // wave-uniform: scores and labels matter only where the boxes overlap enough
                    asm volatile("" ::: "memory");  // keeps this a branch
                    if (ties_ignore) word &= __ballot(c_score > v_score[k]);
                    if (labelled) word &= __ballot(c_class == v_class[k]);
                }
                if (kPretest && word != 0) {  // wave-uniform: some pair of the row may reach the threshold
                    asm volatile("" ::: "memory");  // keeps this a branch
                    const float denom = (v_area[k] + c_area) - inter;
                    unsigned long long maybe = word;
                    if (pretest) maybe &= __ballot(inter >= denom * c_lo);
                    if (maybe != 0) {
                        asm volatile("" ::: "memory");
                        maybe &= __ballot((double)inter >= boundary * (double)denom);
                    }
                    word = maybe;
                }
                words[k] = word;
            }
#pragma unroll
            for (int k = 0; k < kGroup; ++k)
                grp_bits |= (unsigned)((words[k] | (0ull - words[k])) >> 63) << k;  // (word != 0) << k in scalar arithmetic
            if (WRITE_MASK) {
#pragma unroll
                for (int k = 0; k < kGroup; ++k) {
                    if (words[k] != 0) {  // wave-uniform
                        asm volatile("" ::: "memory");  // keeps this a branch (otherwise the move is made for every row)
                        const bool mine = (lane == kGroup * grp + k);
                        w_lo = mine ? (unsigned)words[k] : w_lo;
                        w_hi = mine ? (unsigned)(words[k] >> 32) : w_hi;
                    }
                }
            } else {
                lane_hit |= ((lane / kGroup) == grp) ? ((grp_bits >> (lane % kGroup)) & 1u) : 0u;
            }
        }
        const int row = tr * kTile + lane;
        if (WRITE_MASK) {
            unsigned long long out = ((unsigned long long)w_hi << 32) | w_lo;
            if (row >= n_f) out = 0;
            mask[(size_t)f * ((size_t)(n_pad / kTile) * n_pad) + (size_t)tc * n_pad + row] = out;
        } else {
            if (lane_hit && row < n_f) keep_out[(size_t)f * n_max + order[(size_t)f * n_max + row]] = 0;
        }
    };
    for (; tr < tr_end; ++tr) {
        if (tr == tc) tile(std::true_type());
        else tile(std::false_type());
    }
}
