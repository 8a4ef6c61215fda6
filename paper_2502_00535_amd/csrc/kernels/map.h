// Part of nms_kernels.hip (included there, inside its anonymous namespace): map step: pair tests on the ranked lower triangle, mask-writing and fused (row reduction folded in) forms.
#pragma once

// ----------------------------------------------------------------------------- map

// Work units and their numbering: nms_triangle_unit / nms_triangle_units in nms_host_logic.h.
constexpr int kMapWaves = 4;  // wavefronts (tiles) per workgroup

// State a wavefront carries through the 64 rows of a tile.
struct TileState {
    unsigned lane_hit = 0;           // fused form: lane r = 1 when row r has an eliminator in this tile
    unsigned w_lo = 0, w_hi = 0;     // mask form: lane r collects the 64-bit word of row r
};

// The 64 rows of a tile: victim r (wave-uniform, fetched with scalar loads) against
// the 64 outranking boxes held one per lane.  The ballot of the compare is the
// elimination word of row r.  Rows go in 4 groups of 16 in a real loop, so that at
// most 64 victim SGPRs are live at a time.
// Which evaluation of the pair test a tile uses.
enum { kPairExact = 0, kPairFast = 1, kPairFastYScaled = 2, kPairFastLateScaled = 3 };

// For kPairFastYScaled, vb/cb hold y * NMS_YSCALE, c_T is NMS_YSCALE * T and y_one is
// NMS_YSCALE in a vector register; for kPairFastLateScaled vb/cb are the plain boxes, c_T and
// y_one as for kPairFastYScaled.
template <int PAIR, bool WRITE_MASK, bool DIAG>
__device__ __forceinline__ void tile_sweep(const float4 *__restrict__ vb, const float4 cb, float c_area, float c_T,
                                           float y_one, const NmsThetaConst &th, int lane, TileState &st)
{
    // Rows go in groups of kGroup: the group's victims are fetched together (their scalar
    // loads issue back to back) and its words are formed without any branch in between.
    constexpr int kGroup = WRITE_MASK ? 8 : 16;
#pragma unroll 1
    for (int grp = 0; grp < kTile / kGroup; ++grp) {
        const float4 *__restrict__ vg = vb + kGroup * grp;
        unsigned grp_bits = 0;  // wave-uniform: bit k = row kGroup*grp+k has an eliminator
        unsigned long long words[kGroup];
#pragma unroll
        for (int k = 0; k < kGroup; ++k) {
            const int r = kGroup * grp + k;
            const float4 v = vg[k];
            bool hit;
            if (PAIR == kPairFastYScaled)
                hit = nms_eliminates_fast_yscaled(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, c_T, y_one);
            else if (PAIR == kPairFastLateScaled)
                hit = nms_eliminates_fast_latescaled(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, c_T, y_one);
            else if (PAIR == kPairFast)
                hit = nms_eliminates_fast(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, c_T);
            else
                hit = nms_eliminates_exact(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, c_area, th.theta);
            unsigned long long word = __ballot(hit);
            if (DIAG) word &= (1ull << r) - 1ull;  // only better-ranked boxes eliminate
            words[k] = word;
            grp_bits |= (word != 0 ? 1u : 0u) << k;
        }
        if (WRITE_MASK) {
            // lane r collects the word of row r.  Most rows of most tiles have no eliminator:
            // the move sits behind a wave-uniform branch.
#pragma unroll
            for (int k = 0; k < kGroup; ++k) {
                if (words[k] != 0) {
                    asm volatile("" ::: "memory");  // keeps this a branch (otherwise the move is made for every row)
                    const int r = kGroup * grp + k;
                    const bool mine = (lane == r);
                    st.w_lo = mine ? (unsigned)words[k] : st.w_lo;
                    st.w_hi = mine ? (unsigned)(words[k] >> 32) : st.w_hi;
                }
            }
        } else {
            st.lane_hit |= ((lane >> 4) == grp) ? ((grp_bits >> (lane & 15)) & 1u) : 0u;
        }
    }
}

// One wavefront = one unit: a column tile against up to kSuper victim tiles, so the
// per-lane set-up (loads, threshold) is paid once per 4 x 64 rows.  WRITE_MASK: store each tile's 64 words (mask
// layout of nms.h).  Otherwise: fold the row reduction in and clear keep_out of every
// victim that some lane eliminates (keep_out was preset to 1 by the rank step; all
// writers store the same 0, so concurrent tiles need no atomics).
template <bool FAST, bool WRITE_MASK, int kSuper>
__global__ void __launch_bounds__(kMapWaves * 64)
map_tile_kernel(const float *__restrict__ sorted5, const int32_t *__restrict__ counts, int n_max, int n_pad,
                int tiles, int tile_blocks, int frames, int xcd_frames, NmsThetaConst th,
                unsigned long long *__restrict__ mask, const int32_t *__restrict__ order,
                uint8_t *__restrict__ keep_out, const float4 *__restrict__ ysc, const unsigned *__restrict__ ytile)
{
    const int lane = threadIdx.x & 63;
    int f, bx;
    if (xcd_frames) {
        // Workgroups are dealt to the 8 XCDs round-robin by linear id, and each XCD has its
        // own L2.  Give all tiles of a frame to one XCD (frame f -> XCD f mod 8) so that the
        // frame's box table is fetched from HBM once instead of once per XCD.
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
    const int tiles_f = (n_f + kTile - 1) / kTile;  // tile rows that hold boxes of this frame
    int tr = kSuper * sr > tc ? kSuper * sr : tc;
    int tr_end = kSuper * sr + kSuper < tiles_f ? kSuper * sr + kSuper : tiles_f;
    if (tr >= tr_end) return;

    const float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    const float4 *box4 = reinterpret_cast<const float4 *>(sorted_f);
    const float *area = sorted_f + 4 * (size_t)n_pad;

    // outranking box of this lane, and the float32 its intersections are compared with
    const float4 cb = box4[tc * kTile + lane];
    const float c_area = area[tc * kTile + lane];
    const float c_T = FAST ? nms_pair_threshold(c_area, th.m) : 0.0f;

    // y-scaled form (fast threshold, and the caller has the scaled table and the tile flags
    // of the rank step: the whole-path calls do, the stand-alone map step does not): usable
    // for a tile pair when the rank step flagged both tiles regular.  The pointers are formed
    // unconditionally so that the victims' loads stay scalar loads.
    constexpr bool kScaled = FAST;
    const float4 *__restrict__ ysc4 = ysc + (size_t)f * n_pad;
    const unsigned *__restrict__ ytile_f = ytile + (size_t)f * (n_pad / kTile);
    bool c_regular = false;
    if (kScaled && ysc != nullptr) c_regular = ytile_f[tc] != 0;
    const float4 cbs = make_float4(cb.x, cb.y * NMS_YSCALE, cb.z, cb.w * NMS_YSCALE);
    const float c_Ts = c_T * NMS_YSCALE;
    float y_one;  // NMS_YSCALE in a vector register (opaque to the compiler so it stays there)
    asm volatile("v_mov_b32 %0, 0x38800000" : "=v"(y_one));
    // The mask-writing kernel without the table (the stand-alone map step), or on a tile outside
    // the table's range: the late-scaled form, when every outranking box of this column tile is at
    // most 2^14 high.  (Not in the fused kernel: the table form covers it, and the third variant
    // cost it 1 % through its code size.)
    constexpr bool kLate = FAST && WRITE_MASK;
    const bool late_ok = kLate && __ballot(!nms_extent_fits_late_scaling(cb.y, cb.w)) == 0ull;

    for (; tr < tr_end; ++tr) {
        TileState st;
        if (kScaled && c_regular && ytile_f[tr] != 0) {
            const float4 *vb = ysc4 + tr * kTile;  // victims: wave-uniform addresses -> scalar loads
            if (tr == tc)
                tile_sweep<kPairFastYScaled, WRITE_MASK, true>(vb, cbs, c_area, c_Ts, y_one, th, lane, st);
            else
                tile_sweep<kPairFastYScaled, WRITE_MASK, false>(vb, cbs, c_area, c_Ts, y_one, th, lane, st);
        } else if (kLate && late_ok) {
            const float4 *vb = box4 + tr * kTile;
            if (tr == tc)
                tile_sweep<kPairFastLateScaled, WRITE_MASK, true>(vb, cb, c_area, c_Ts, y_one, th, lane, st);
            else
                tile_sweep<kPairFastLateScaled, WRITE_MASK, false>(vb, cb, c_area, c_Ts, y_one, th, lane, st);
        } else {
            const float4 *vb = box4 + tr * kTile;
            if (tr == tc)
                tile_sweep<FAST ? kPairFast : kPairExact, WRITE_MASK, true>(vb, cb, c_area, c_T, y_one, th, lane, st);
            else
                tile_sweep<FAST ? kPairFast : kPairExact, WRITE_MASK, false>(vb, cb, c_area, c_T, y_one, th, lane, st);
        }

        const int row = tr * kTile + lane;
        if (WRITE_MASK) {
            unsigned long long out = ((unsigned long long)st.w_hi << 32) | st.w_lo;
            if (row >= n_f) out = 0;  // padding rows of the last tile
            mask[(size_t)f * ((size_t)(n_pad / kTile) * n_pad) + (size_t)tc * n_pad + row] = out;
        } else {
            if (st.lane_hit && row < n_f)
                keep_out[(size_t)f * n_max + order[(size_t)f * n_max + row]] = 0;
        }
    }
}

// ----------------------------------------------------------------------------- fused map, lane = victim

// The whole-path calls do not need the mask, only "does row r have an eliminator".  With the
// roles exchanged -- lane = VICTIM r of a tile row (its box in registers), the outranking box c
// wave-uniform, fetched with scalar loads together with its precomputed decision threshold -- the
// compare's lane mask is, for one outranking box, the set of victims it eliminates, and the row
// reduction is a running OR of those masks: one scalar instruction per 64 pair tests instead
// of three (test for zero, select a bit, merge), and at the end lane r itself holds the answer
// for row r, so a victim is written at most once per work unit and no threshold has to be worked
// out per lane.  The ten VALU instructions of the pair test are the same.
//
// caux: per outranking box, NMS_YSCALE * T (written by the rank step; the unscaled forms multiply
// it back up, a power of two) or, for thresholds that take the literal division, the area.
// Wave-uniform reads of tables that a previous kernel wrote and this one never writes: through
// the constant address space, so that they are scalar loads whatever else the kernel loads.
typedef const __attribute__((address_space(4))) float *nms_uniform_float_ptr;

// Which victims of the wavefront an outranking box may eliminate at all: every lane (the tile of
// outranking boxes lies wholly before the victims), the lanes behind it in the same tile, or --
// lanes that hold victims of arbitrary ranks -- the lanes whose victim is ranked behind it.
enum { kMaskNone = 0, kMaskDiagonal = 1, kMaskByRank = 2 };

// r_lane: rank of the lane's victim, c_base: rank of the tile's first outranking box (kMaskByRank only).
// The tile's boxes are taken in groups of kFusedGroup, groups [grp_begin, grp_end).
constexpr int kFusedGroup = 8;  // outranking boxes fetched together: 40 SGPRs

template <int PAIR, int MASK>
__device__ __forceinline__ unsigned long long fused_candidates(const float4 *__restrict__ cb,
                                                               const float *__restrict__ caux, const float4 vb,
                                                               float y_one, float theta, int r_lane, int c_base,
                                                               int grp_begin = 0, int grp_end = kTile / kFusedGroup)
{
    unsigned long long acc = 0;
    constexpr int kGroup = kFusedGroup;
#pragma unroll 1
    for (int grp = grp_begin; grp < grp_end; ++grp) {
        const nms_uniform_float_ptr cg = (nms_uniform_float_ptr)(uintptr_t)(cb + kGroup * grp);
        const nms_uniform_float_ptr ag = (nms_uniform_float_ptr)(uintptr_t)(caux + kGroup * grp);
#pragma unroll
        for (int k = 0; k < kGroup; ++k) {
            const float4 c = make_float4(cg[4 * k], cg[4 * k + 1], cg[4 * k + 2], cg[4 * k + 3]);
            const float a = ag[k];
            bool hit;
            if (PAIR == kPairFastYScaled)
                hit = nms_eliminates_fast_yscaled(vb.x, vb.y, vb.z, vb.w, c.x, c.y, c.z, c.w, a, y_one);
            else if (PAIR == kPairFast)
                hit = nms_eliminates_fast(vb.x, vb.y, vb.z, vb.w, c.x, c.y, c.z, c.w, a * (1.0f / NMS_YSCALE));
            else
                hit = nms_eliminates_exact(vb.x, vb.y, vb.z, vb.w, c.x, c.y, c.z, c.w, a, theta);
            unsigned long long word = __ballot(hit);
            const int ci = kGroup * grp + k;
            if (MASK == kMaskDiagonal) word &= ci == kTile - 1 ? 0ull : (~0ull << (ci + 1));
            if (MASK == kMaskByRank) word &= __ballot(r_lane > c_base + ci);
            acc |= word;
        }
    }
    return acc;
}

// The same with the next group's scalar loads in flight while a group is worked on, for launches
// that leave a SIMD with one or two wavefronts and nobody else to cover a load's latency (the
// two-launch route's second launch).  Groups of four (two buffers of 20 scalar registers).  Scalar
// loads may complete out of order, so a wait for one buffer waits for all loads issued before it:
// the next group is requested only after the current one has arrived.
template <int PAIR, int MASK>
__device__ __forceinline__ unsigned long long fused_candidates_ahead(const float4 *__restrict__ cb,
                                                                     const float *__restrict__ caux, const float4 vb,
                                                                     float y_one, float theta, int r_lane, int c_base)
{
    constexpr int kGroup = 4;
    constexpr int kGroups = kTile / kGroup;
    unsigned long long acc = 0;
    float4 c[2][kGroup];
    float a[2][kGroup];
    auto fetch = [&](int buf, int grp) __attribute__((always_inline)) {
        const nms_uniform_float_ptr cg = (nms_uniform_float_ptr)(uintptr_t)(cb + kGroup * grp);
        const nms_uniform_float_ptr ag = (nms_uniform_float_ptr)(uintptr_t)(caux + kGroup * grp);
#pragma unroll
        for (int k = 0; k < kGroup; ++k) {
            c[buf][k] = make_float4(cg[4 * k], cg[4 * k + 1], cg[4 * k + 2], cg[4 * k + 3]);
            a[buf][k] = ag[k];
        }
    };
    auto work = [&](int buf, int grp) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < kGroup; ++k) {
            const float4 cc = c[buf][k];
            const float aa = a[buf][k];
            bool hit;
            if (PAIR == kPairFastYScaled)
                hit = nms_eliminates_fast_yscaled(vb.x, vb.y, vb.z, vb.w, cc.x, cc.y, cc.z, cc.w, aa, y_one);
            else if (PAIR == kPairFast)
                hit = nms_eliminates_fast(vb.x, vb.y, vb.z, vb.w, cc.x, cc.y, cc.z, cc.w, aa * (1.0f / NMS_YSCALE));
            else
                hit = nms_eliminates_exact(vb.x, vb.y, vb.z, vb.w, cc.x, cc.y, cc.z, cc.w, aa, theta);
            unsigned long long word = __ballot(hit);
            const int ci = kGroup * grp + k;
            if (MASK == kMaskDiagonal) word &= ci == kTile - 1 ? 0ull : (~0ull << (ci + 1));
            if (MASK == kMaskByRank) word &= __ballot(r_lane > c_base + ci);
            acc |= word;
        }
    };
    fetch(0, 0);
#pragma unroll 1
    for (int grp = 0; grp < kGroups; grp += 2) {
        asm volatile("" ::"s"(a[0][kGroup - 1]));  // buffer 0 has arrived ...
        __builtin_amdgcn_sched_barrier(0);
        fetch(1, grp + 1);                           // ... request the next group, then work
        __builtin_amdgcn_sched_barrier(0);
        work(0, grp);
        asm volatile("" ::"s"(a[1][kGroup - 1]));
        __builtin_amdgcn_sched_barrier(0);
        fetch(0, grp + 2 < kGroups ? grp + 2 : 0);  // (the last request is not used)
        __builtin_amdgcn_sched_barrier(0);
        work(1, grp + 1);
    }
    return acc;
}

// One wavefront = one unit: a victim tile row tr against up to kSuper tiles of outranking boxes
// tc <= tr.  Units are numbered as in nms_triangle_unit with both tile indices counted from the
// far end (u = T-1-tr, v = T-1-tc, v >= u, the v of a unit share v / kSuper).  keep_out was preset
// to 1 by the rank step; every writer stores 0, so concurrent units need no atomics.
template <bool FAST, int kSuper>
__global__ void __launch_bounds__(kMapWaves * 64)
map_fused_kernel(const float *__restrict__ sorted5, const int32_t *__restrict__ counts, int n_max, int n_pad,
                 int tiles, int tile_blocks, int frames, int xcd_frames, NmsThetaConst th,
                 const int32_t *__restrict__ order, uint8_t *__restrict__ keep_out,
                 const float4 *__restrict__ ysc, const unsigned *__restrict__ ytile, const float *__restrict__ tsc)
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
    const int T = n_pad / kTile;
    int sr, u;
    nms_triangle_unit<kSuper>(g, sr, u);
    const int tr = T - 1 - u;                       // victim tile row
    const int tiles_f = (n_f + kTile - 1) / kTile;  // tile rows that hold boxes of this frame
    if (tr >= tiles_f) return;
    int v = kSuper * sr > u ? kSuper * sr : u;
    const int v_end = kSuper * sr + kSuper < T ? kSuper * sr + kSuper : T;

    const float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    const float4 *__restrict__ box4 = reinterpret_cast<const float4 *>(sorted_f);
    const float *__restrict__ area = sorted_f + 4 * (size_t)n_pad;
    const float4 *__restrict__ ysc4 = ysc + (size_t)f * n_pad;
    const unsigned *__restrict__ ytile_f = ytile + (size_t)f * (n_pad / kTile);
    const float *__restrict__ tsc_f = tsc + (size_t)f * n_pad;

    const int row = tr * kTile + lane;
    const float4 vbs = ysc4[row];  // this lane's victim, y scaled
    const bool r_regular = FAST && ytile_f[tr] != 0;  // the rank step's flag: the tile may take the y-scaled form
    float y_one;  // NMS_YSCALE in a vector register (opaque to the compiler so it stays there)
    asm volatile("v_mov_b32 %0, 0x38800000" : "=v"(y_one));

    unsigned long long acc = 0;
    for (; v < v_end; ++v) {
        const int tc = T - 1 - v;
        if (r_regular && ytile_f[tc] != 0) {
            if (tc == tr)
                acc |= fused_candidates<kPairFastYScaled, kMaskDiagonal>(ysc4 + tc * kTile, tsc_f + tc * kTile, vbs, y_one, th.theta, 0, 0);
            else
                acc |= fused_candidates<kPairFastYScaled, kMaskNone>(ysc4 + tc * kTile, tsc_f + tc * kTile, vbs, y_one, th.theta, 0, 0);
        } else {
            const float4 vb = box4[row];
            const float *caux = FAST ? tsc_f + tc * kTile : area + tc * kTile;
            if (tc == tr)
                acc |= fused_candidates<FAST ? kPairFast : kPairExact, kMaskDiagonal>(box4 + tc * kTile, caux, vb, y_one, th.theta, 0, 0);
            else
                acc |= fused_candidates<FAST ? kPairFast : kPairExact, kMaskNone>(box4 + tc * kTile, caux, vb, y_one, th.theta, 0, 0);
        }
    }
    if (((acc >> lane) & 1ull) && row < n_f) keep_out[(size_t)f * n_max + order[(size_t)f * n_max + row]] = 0;
}
