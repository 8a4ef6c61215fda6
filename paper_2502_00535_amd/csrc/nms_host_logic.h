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
    size_t stage;    // uint64 [frames][n_pad / 64][32] eliminated-victim masks of the two-launch route, only when n_max > sort_chunk
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
    l.stage = p;
    if (n_max > sort_chunk) p += nms_align256((size_t)frames * (size_t)(n_pad / 64) * 32 * sizeof(unsigned long long));
    l.end = p;
    return l;
}

// ---- which kernels a whole-path call runs ------------------------------------------------------
// All four routes return the same keep vector (the paper's rule, section "Algorithm Correctness");
// they differ in what they launch.  Values of nms_route() in the C ABI.
constexpr int kNmsRouteDirect = 0;     // one launch, full n x n pair set with the score test inside (no rank step)
constexpr int kNmsRouteAllPairs = 1;   // rank, then every pair of the ranked triangle
constexpr int kNmsRouteTwoLaunch = 2;  // rank, every victim against the best 2048 ranks, then the live victims only
constexpr int kNmsRouteEarlyExit = 3;  // rank, then stages that drop a victim once it has an eliminator
constexpr int kNmsRouteSmallFrames = 4;  // frames of at most 1024 boxes, or a few of up to 4096: two such stages in one launch, no sort

// Frames small enough that launch latency, not arithmetic, decides: one launch of the
// direct form instead of rank + map.  (Twice the pairs and two more compares per pair:
// about 2.5x the VALU work of the ranked triangle.)
// The crossover in GPU time sits near 2^25 pair slots per batch and moves with the frame size,
// because the rank step it saves does (15 us at 1024 boxes, 23 us at 4096): measured 24 to 32
// frames of 1024 boxes, 8 to 12 of 2048, 3 to 4 of 4096.
NMS_HD bool nms_use_direct_form(int n_max, int frames)
{
    const long long slots = (long long)frames * n_max * n_max;
    const long long limit = n_max > 2048 ? (3ll << 24) : (n_max > 512 && n_max <= 1024 ? (3ll << 23) : (1ll << 25));
    return n_max <= 4096 && slots <= limit;
}

// Frames beyond sort_chunk boxes, a few of them (2^27 to 2^31 pair slots: one frame of 16,384
// boxes, four of them, eight of 8192): two launches with the decided victims dropped in between.
// Measured on dense crowd scenes, whole call: 1 x 16,384 38 us (all pairs 50), 4 x 16,384 82 us
// (all pairs 143, the early-exit kernels 98), 1 x 32,400 94 us (137 / 108); from 2^31 slots on
// the early-exit kernels are quicker (16 x 16,384: 200 us against 262).
NMS_HD bool nms_use_two_launches(int n_max, int frames, int sort_chunk)
{
    const long long slots = (long long)frames * n_max * n_max;
    return n_max > sort_chunk && slots >= (1ll << 27) && slots < (1ll << 31);
}

// Large batches of frames of a thousand boxes or more: the route that stops testing a victim
// once it has an eliminator returns the same keep vector 1.3 to 3.3 times sooner on clustered
// detections (what a detector emits) and 0.7 to 1.0 times as fast when almost nothing is
// eliminated (measured on 32 to 1024 frames of 1024 to 4096 boxes).  Frames of 512 boxes or
// fewer never gain: their stages are mostly barriers.  From 2^28 pair slots on (64 x 2048: 40 us
// against 43 for all pairs; 64 x 1536, below: 38 against 33).  Frames beyond sort_chunk boxes take
// it from 2^31 pair slots on (below that the two launches are quicker).  (nms_route_for asks
// nms_use_small_frames first, which takes the batches of frames of up to 1024 boxes and small
// batches of longer ones.)
NMS_HD bool nms_use_early_exit(int n_max, int frames, int sort_chunk)
{
    const long long slots = (long long)frames * n_max * n_max;
    return n_max > sort_chunk ? slots >= (1ll << 31) : (n_max > 1024 && slots >= (1ll << 28));
}

// Workgroups that share a frame in the small-frames kernels (each builds the tables of the whole
// frame and takes every parts-th tile of victims; a share is at most 16 tiles, and more workgroups
// than tiles would only build tables).  Frames of up to 1024 boxes: doubled while that leaves at most
// one workgroup per compute unit (256), and once more -- two workgroups fit a compute unit -- as
// long as a share keeps four tiles of victims (measured: 256 x 1024 31.6 -> 28.4 us, 256 x 768
// 36.3 -> 26.5; with two-tile shares, 64 x 1024 12.4 -> 13.9).  Longer frames: one workgroup per
// compute unit (their tables fill its LDS), as many as that allows.
NMS_HD int nms_small_frames_parts(int frames, int n_max)
{
    const int tiles = (n_max + 63) / 64;
    const int most = tiles < 64 ? tiles : 64;  // a workgroup without a tile of victims would only build tables
    int parts = (tiles + 15) / 16;
    if (n_max <= 512) {  // workgroups of 512 threads, up to four on a compute unit
        parts = 1;
        while (parts * 2 <= tiles && (long long)frames * parts * 2 <= 512) parts *= 2;
        return parts;
    }
    if (n_max > 1024) {
        const int fit = 256 / (frames < 256 ? frames : 256);
        return fit > most ? most : (fit < parts ? parts : fit);
    }
    while (parts * 2 <= most && (long long)frames * parts * 2 <= 256) parts *= 2;
    while (parts * 2 <= most && (long long)frames * parts * 2 <= 512 && tiles / (parts * 2) >= 4) parts *= 2;
    return parts;
}

// Frames of 513 to 1024 boxes, ten or more of them (longer and shorter frames: inside): one launch without a sort, in which a
// workgroup of 1024 threads tests every victim of its frame against the two best-ranked of every
// sixteen input elements and the victims still alive against the whole frame (clustered detections,
// whole call: 64 x 1024 11.8 us, all pairs 20.8; 256 x 1024 28.4, early exit 34.5, all pairs 43.2;
// 2048 x 1024 155, early exit 197; 128 x 640 17.6, all pairs 20.3).  Its workgroups are 1024 threads
// and its tables 1024 rows whatever the frame size, so short frames gain nothing (256 x 512: 19.3
// against 20.4; 192 x 576: 26.0 against 21.7), and between 256 and 512 frames the workgroups beyond
// one per compute unit share a compute unit with another (300 x 768: 40.8 against 37.7; 300 x 1024:
// 45.0 against 47.9).  In tiles of 64 boxes per frame:
NMS_HD bool nms_use_small_frames(int n_max, int frames)
{
    const int tiles = (n_max + 63) / 64;
    if (n_max > 1024) {
        // Frames of 1025 to 4096 boxes (two or four elements per thread), a few of them.  Below 2^25 pair slots the
        // direct form is quicker (4 x 2048: 9.5 us against 10.6; the tables cost 4 us before the first pair test).
        // Above that the kernel wins while a workgroup's share stays at four tiles of victims (five beyond 2048
        // boxes) with one workgroup per compute unit: 8 x 2048 11 us against 17 (direct), 32 x 2048 25 against 30
        // (all pairs), 4 x 4096 15 against 29, 16 x 4096 33 against 40 (early exit), 40 x 1536 24.5 against 26.4;
        // 44 x 1536 31.5 against 28.5, 56 x 1100 30.8 against 25.0, 29 x 3000 47.8 against 48.1.
        if (n_max > 4096 || frames > 256 || (long long)frames * n_max * n_max < (1ll << 25)) return false;
        const int parts = nms_small_frames_parts(frames, n_max);
        return (tiles + parts - 1) / parts <= (n_max > 2048 ? 5 : 4);
    }
    // frames of 449 to 512 boxes (workgroups of 512 threads), many of them: 256 x 512 16.3 us against 20.1 for all pairs,
    // 2048 x 512 72 against 97; 128 x 512 13.2 against 14.4 (direct); shorter frames or fewer gain nothing (512 x 384: 25.0
    // against 23.9; 64 x 512: 8.9 against 8.6)
    if (n_max <= 512) return tiles == 8 && frames >= 128;
    // against the direct form, where that would be taken (10 to 32 frames: 12 x 1024 7.1 us against 8.5, 24 x 1024 8.2
    // against 15.4, 32 x 768 8.5 against 9.4; 8 x 1024 7.0 against 6.3, 16 x 768 7.2 against 6.2, 32 x 576 8.8 against 8.0)
    if (nms_use_direct_form(n_max, frames)) return tiles >= 10 && (long long)frames * n_max * n_max > (5ll << 21);
    if (frames <= 128) return tiles >= 9;
    if (frames <= 256) return tiles >= 11;
    if (frames < 512) return tiles >= 15;
    return tiles >= 11;
}

// The route of the automatic whole-path call for a batch shape (1 <= n_max, 1 <= frames).
NMS_HD int nms_route_for(int n_max, int frames, int sort_chunk)
{
    if (nms_use_small_frames(n_max, frames)) return kNmsRouteSmallFrames;
    if (nms_use_direct_form(n_max, frames)) return kNmsRouteDirect;
    if (nms_use_early_exit(n_max, frames, sort_chunk)) return kNmsRouteEarlyExit;
    if (nms_use_two_launches(n_max, frames, sort_chunk)) return kNmsRouteTwoLaunch;
    return kNmsRouteAllPairs;
}
