// HIP kernels (gfx950, wave64) and the C ABI of the data-parallel NMS library.
//
// Steps (names follow the paper: D = detections, B = boolean matrix, V = survivors):
//   rank     total order on scores (Algorithm 1's guard "D[i].s < D[j].s", hoisted)
//   map      Algorithm 1 on the ranked lower triangle, one wavefront per 64x64 tile
//   reduce   Algorithm 2's row AND (here: row OR of elimination bits == 0)
//   fused    map with the row reduction folded in; no mask reaches memory
//
// Wave layout of the map step: lane = outranking box c of the tile's column block
// (its box and its per-box decision threshold live in VGPRs for the whole tile); the
// victim row r is wave-uniform and is fetched with scalar loads, so each victim costs
// 4 SGPRs and the 11 VALU instructions of the pair test.  The compare's lane mask IS the 64-bit
// elimination word of (row r, column block): no cross-lane work is needed to form it.
#include <hip/hip_runtime.h>

#include <math.h>
#include <string.h>

#include "../../include/nms.h"
#include "nms_pair.h"

namespace {

constexpr int kTile = NMS_TILE;
constexpr int kChunk = NMS_SORT_CHUNK;
constexpr unsigned long long kSentinel = ~0ull;

__device__ __forceinline__ int frame_count(const int32_t *counts, int f, int n_max)
{
    if (counts == nullptr) return n_max;
    int c = counts[f];
    return c < 0 ? 0 : (c > n_max ? n_max : c);
}

// ----------------------------------------------------------------------------- rank

// Unique ascending 64-bit key: better score first, then lower index.
__device__ __forceinline__ unsigned long long rank_key(float score, unsigned idx)
{
    unsigned u = __float_as_uint(score);
    if (u == 0x80000000u) u = 0u;  // -0.0 ties with +0.0
    unsigned asc = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
    return ((unsigned long long)(~asc) << 32) | idx;
}

// Rank-ordered row r: the box and its area, and (fused path only, ysc != nullptr) the same
// box with y multiplied by NMS_YSCALE.  Returns whether the box may use the y-scaled form.
__device__ __forceinline__ bool emit_ranked_box(const float4 b, int idx, int r, int n_pad,
                                               int32_t *order_f, float *sorted_f, float4 *ysc_f)
{
    order_f[r] = idx;
    reinterpret_cast<float4 *>(sorted_f)[r] = b;
    sorted_f[4 * (size_t)n_pad + r] = nms_box_area(b.x, b.y, b.z, b.w);
    if (ysc_f != nullptr) ysc_f[r] = make_float4(b.x, b.y * NMS_YSCALE, b.z, b.w * NMS_YSCALE);
    return nms_y_regular(b.y) && nms_y_regular(b.w);
}

__device__ __forceinline__ void emit_padding_row(int r, int n_pad, float *sorted_f, float4 *ysc_f)
{
    reinterpret_cast<float4 *>(sorted_f)[r] = make_float4(0.f, 0.f, 0.f, 0.f);
    sorted_f[4 * (size_t)n_pad + r] = 1.0f;  // the one-pixel box (0,0,0,0): never divides by zero
    if (ysc_f != nullptr) ysc_f[r] = make_float4(0.f, 0.f, 0.f, 0.f);
}

// Inclusive prefix sum over the 64 lanes of a wavefront with DPP: shifts by 1, 2, 4, 8 inside
// each row of 16 lanes (lanes shifted in from outside a row read 0), then lane 15 of each row
// broadcast into the next row (rows 1 and 3), then lane 31 into rows 2 and 3.
__device__ __forceinline__ unsigned wave_inclusive_sum(unsigned x)
{
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, true);  // row_shr:1
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, true);  // row_shr:2
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, true);  // row_shr:4
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, true);  // row_shr:8
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x142, 0xa, 0xf, false); // row_bcast:15 into rows 1, 3
    x += (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x143, 0xc, 0xf, false); // row_bcast:31 into rows 2, 3
    return x;
}

// Stable LSD radix sort of the P = 4 * blockDim.x (key, index) pairs of a workgroup, eight
// bits per pass, four passes.  Element e = 256 * wave + 64 * q + lane is register q of its
// thread.  Stability is what makes 32-bit keys enough: elements start in index order, so
// equal scores keep the lower index first (the tie rule) without the index taking part in
// any compare.  Per pass:
//   - every wavefront ranks its 256 elements among themselves: for q = 0..3 in turn, the
//     lanes that hold the same digit find each other with eight ballots, take their place
//     after the elements of earlier q with that digit (running per-wavefront histogram in
//     LDS, touched by its own wavefront only) and the group's first lane bumps the histogram;
//   - the histograms are turned into start offsets per (digit, wavefront): column sums,
//     then one wavefront scans the 256 digit totals;
//   - every element goes to start + place in `buf`, and the threads read their elements back.
// After the last pass `buf` holds ((key << 32) | index) in sorted order.
__device__ __forceinline__ void radix_rank_chunk(unsigned (&key)[4], unsigned (&idx)[4], const int (&e)[4],
                                                 unsigned long long *buf, unsigned *hist, unsigned *tot,
                                                 unsigned *dbase)
{
    const int tid = threadIdx.x;
    const int nth = blockDim.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int W = nth >> 6;
    unsigned *myhist = hist + wave * 256;
#pragma unroll 1
    for (int shift = 0; shift < 32; shift += 8) {
        for (int i = lane; i < 256; i += 64) myhist[i] = 0;
        unsigned place[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned d = (key[q] >> shift) & 255u;
            unsigned m_lo = ~0u, m_hi = ~0u;  // lanes whose digit equals mine
#pragma unroll
            for (int b = 0; b < 8; ++b) {
                const unsigned all = 0u - ((d >> b) & 1u);  // all ones if my bit b is set
                const unsigned long long set = __ballot(all != 0);
                m_lo &= ~((unsigned)set ^ all);
                m_hi &= ~((unsigned)(set >> 32) ^ all);
            }
            const unsigned below = __builtin_amdgcn_mbcnt_hi(m_hi, __builtin_amdgcn_mbcnt_lo(m_lo, 0u));
            const unsigned total = __popc(m_lo) + __popc(m_hi);
            const unsigned base = myhist[d];
            if (below == 0) myhist[d] = base + total;
            place[q] = base + below;
        }
        __syncthreads();
        for (int d = tid; d < 256; d += nth) {
            // the counts of digit d in every wavefront (all reads issued together), then their running sums
            unsigned t[kChunk / 256];
#pragma unroll
            for (int w = 0; w < kChunk / 256; ++w) t[w] = w < W ? hist[w * 256 + d] : 0u;
            unsigned run = 0;
#pragma unroll
            for (int w = 0; w < kChunk / 256; ++w) {
                if (w < W) hist[w * 256 + d] = run;
                run += t[w];
            }
            tot[d] = run;
        }
        __syncthreads();
        if (wave == 0) {
            const unsigned a0 = tot[4 * lane], a1 = tot[4 * lane + 1], a2 = tot[4 * lane + 2], a3 = tot[4 * lane + 3];
            const unsigned sum = a0 + a1 + a2 + a3;
            const unsigned incl = wave_inclusive_sum(sum);
            const unsigned excl = incl - sum;
            dbase[4 * lane] = excl;
            dbase[4 * lane + 1] = excl + a0;
            dbase[4 * lane + 2] = excl + a0 + a1;
            dbase[4 * lane + 3] = excl + a0 + a1 + a2;
        }
        __syncthreads();
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned d = (key[q] >> shift) & 255u;
            const unsigned dest = dbase[d] + myhist[d] + place[q];
            buf[dest] = ((unsigned long long)key[q] << 32) | idx[q];
        }
        __syncthreads();
        if (shift < 24) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const unsigned long long v = buf[e[q]];
                key[q] = (unsigned)(v >> 32);
                idx[q] = (unsigned)v;
            }
        }
    }
}

// One workgroup ranks one chunk of up to kChunk boxes of one frame: P = 4 * blockDim.x
// elements (P a multiple of 256, 256..4096), four per thread, sorted by radix_rank_chunk.
// With a single chunk the kernel also writes order / sorted5 (and, for the fused path,
// presets keep_out); with several chunks it leaves the chunk's sorted keys in `keys_ws`
// for the merge kernel.
__global__ void __launch_bounds__(1024)
rank_chunk_kernel(const float *__restrict__ boxes, const float *__restrict__ scores,
                  const int32_t *__restrict__ counts, int n_max, int n_pad, int n_chunks,
                  int32_t *__restrict__ order, float *__restrict__ sorted5,
                  unsigned long long *__restrict__ keys_ws, uint8_t *__restrict__ keep_preset,
                  float4 *__restrict__ ysc, unsigned *__restrict__ ytile)
{
    __shared__ unsigned long long keys[kChunk];
    __shared__ unsigned hist[(kChunk / 256) * 256];  // one row of 256 digit counts per wavefront
    __shared__ unsigned tot[256];
    __shared__ unsigned dbase[256];
    const int f = blockIdx.y;
    const int chunk = blockIdx.x;
    const int tid = threadIdx.x;
    const int nth = blockDim.x;
    const int lane = tid & 63;
    const int n_f = frame_count(counts, f, n_max);
    const int base = chunk * kChunk;
    int cnt = n_f - base;
    cnt = cnt < 0 ? 0 : (cnt > kChunk ? kChunk : cnt);
    const float *scores_f = scores + (size_t)f * n_max;
    int e[4];
    unsigned long long K[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        e[q] = (tid >> 6) * 256 + q * 64 + lane;
        K[q] = (e[q] < cnt) ? rank_key(scores_f[base + e[q]], (unsigned)(base + e[q])) : kSentinel;
    }

    unsigned key32[4], index[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        key32[q] = (unsigned)(K[q] >> 32);
        index[q] = (unsigned)K[q];
    }
    radix_rank_chunk(key32, index, e, keys, hist, tot, dbase);  // ends with a barrier; keys[] is sorted

    const float *boxes_f = boxes + (size_t)f * n_max * 4;
    int32_t *order_f = order + (size_t)f * n_max;
    float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    float4 *ysc_f = ysc ? ysc + (size_t)f * n_pad : nullptr;
    unsigned *ytile_f = ytile ? ytile + (size_t)f * (n_pad / kTile) : nullptr;
    if (n_chunks == 1) {
        // n_pad <= 4 * nth: at most four ranks per thread, r = tid + q * nth (a wavefront covers 64
        // consecutive ranks = one tile per q).  The four gathers are issued before anything is
        // stored, so the thread waits for memory once, not once per rank.
        float4 b[4];
        int idx[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int r = tid + q * nth;
            idx[q] = r < n_f ? (int)(unsigned)keys[r] : -1;
            b[q] = idx[q] >= 0 ? reinterpret_cast<const float4 *>(boxes_f)[idx[q]] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int r = tid + q * nth;
            if (r < n_pad) {  // uniform per wavefront (n_pad and nth are multiples of 64)
                bool regular = true;
                if (idx[q] >= 0)
                    regular = emit_ranked_box(b[q], idx[q], r, n_pad, order_f, sorted_f, ysc_f);
                else
                    emit_padding_row(r, n_pad, sorted_f, ysc_f);
                if (ytile_f != nullptr) {
                    const unsigned long long irregular = __ballot(!regular);
                    if (lane == 0) ytile_f[r / kTile] = irregular == 0 ? 1u : 0u;
                }
            }
        }
    } else {
        unsigned long long *kw = keys_ws + (size_t)f * n_pad + base;
        for (int i = tid; i < cnt; i += nth) kw[i] = keys[i];
        // the merge kernel scatters rows, so it can only clear tile flags: preset them here
        if (ytile_f != nullptr && chunk == 0)
            for (int t = tid; t < n_pad / kTile; t += nth) ytile_f[t] = 1u;
    }
    if (keep_preset != nullptr) {
        // fused path: every real box starts as a survivor, slots beyond the count are 0
        uint8_t *kp = keep_preset + (size_t)f * n_max;
        const int hi = (base + kChunk < n_max) ? base + kChunk : n_max;
        for (int i = base + tid; i < hi; i += nth) kp[i] = (i < n_f) ? 1 : 0;
    }
}

// Several chunks: the rank of a key is its position inside its own chunk plus the
// number of smaller keys in every other chunk (keys are unique, so ranks are too).
__global__ void __launch_bounds__(256)
rank_merge_kernel(const float *__restrict__ boxes, const int32_t *__restrict__ counts, int n_max, int n_pad,
                  int n_chunks, const unsigned long long *__restrict__ keys_ws,
                  int32_t *__restrict__ order, float *__restrict__ sorted5,
                  float4 *__restrict__ ysc, unsigned *__restrict__ ytile)
{
    const int f = blockIdx.y;
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= n_pad) return;
    const int n_f = frame_count(counts, f, n_max);
    float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    float4 *ysc_f = ysc ? ysc + (size_t)f * n_pad : nullptr;
    if (e >= n_f) {
        emit_padding_row(e, n_pad, sorted_f, ysc_f);
        return;
    }
    const unsigned long long *kw = keys_ws + (size_t)f * n_pad;
    const unsigned long long key = kw[e];
    const int own = e / kChunk;
    int rank = e - own * kChunk;
    for (int c = 0; c < n_chunks; ++c) {
        if (c == own) continue;
        const int base = c * kChunk;
        int cnt = n_f - base;
        cnt = cnt < 0 ? 0 : (cnt > kChunk ? kChunk : cnt);
        int lo = 0, hi = cnt;  // first position whose key is not smaller
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (kw[base + mid] < key) lo = mid + 1; else hi = mid;
        }
        rank += lo;
    }
    const int idx = (int)(unsigned)key;
    const bool regular = emit_ranked_box(reinterpret_cast<const float4 *>(boxes + (size_t)f * n_max * 4)[idx], idx, rank,
                                         n_pad, order + (size_t)f * n_max, sorted_f, ysc_f);
    // tile flags were preset to 1 by the chunk kernel; concurrent writers all store 0
    if (ytile != nullptr && !regular) ytile[(size_t)f * (n_pad / kTile) + rank / kTile] = 0u;
}

// ----------------------------------------------------------------------------- map

// Work unit of the map step: one column tile tc (64 outranking boxes, held in registers)
// against a "super-row" of kSuper consecutive victim tile rows, i.e. up to kSuper tiles of
// the ranked lower triangle.  Super-row sr has min(kSuper*(sr+1), T) units (tc = 0 .. last
// tile row of the super-row), so the units before super-row sr number
// kSuper * sr*(sr+1)/2.  Linear unit index -> (sr, tc) by integer square root.
// kSuper = 4 amortises the per-lane set-up over 256 rows and is used when the launch has
// plenty of units; kSuper = 1 (one tile per wavefront) keeps small launches balanced.
template <int kSuper>
__device__ __forceinline__ void triangle_unit(int g, int &sr, int &tc)
{
    // largest sr with kSuper*sr*(sr+1)/2 <= g
    int r = (int)((__fsqrt_rn(1.0f + (8.0f / kSuper) * (float)g) - 1.0f) * 0.5f);
    while (kSuper * r * (r + 1) / 2 > g) --r;
    while (kSuper * (r + 1) * (r + 2) / 2 <= g) ++r;
    sr = r;
    tc = g - kSuper * r * (r + 1) / 2;
}

// Number of units for T tile rows.
inline int triangle_units(int T, int super)
{
    const int SR = (T + super - 1) / super;
    return SR == 0 ? 0 : super * (SR - 1) * SR / 2 + T;
}

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
enum { kPairExact = 0, kPairFast = 1, kPairFastYScaled = 2 };

// For kPairFastYScaled, vb/cb hold y * NMS_YSCALE, c_T is NMS_YSCALE * T and y_one is
// NMS_YSCALE in a vector register.
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
    triangle_unit<kSuper>(g, sr, tc);
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

    for (; tr < tr_end; ++tr) {
        TileState st;
        if (kScaled && c_regular && ytile_f[tr] != 0) {
            const float4 *vb = ysc4 + tr * kTile;  // victims: wave-uniform addresses -> scalar loads
            if (tr == tc)
                tile_sweep<kPairFastYScaled, WRITE_MASK, true>(vb, cbs, c_area, c_Ts, y_one, th, lane, st);
            else
                tile_sweep<kPairFastYScaled, WRITE_MASK, false>(vb, cbs, c_area, c_Ts, y_one, th, lane, st);
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

// ----------------------------------------------------------------------------- direct (unranked) form

// The paper's own formulation for small frames: Algorithm 1 on the full n x n grid of
// the UNSORTED input with the score guard evaluated per pair, and Algorithm 2's row
// AND finished inside the workgroup, in one launch (no rank step, no mask, no scratch).
// It evaluates every unordered pair twice and pays two extra compares per pair for the
// guard, so it only wins where launch latency dominates: single frames up to a few
// thousand boxes.
//
// A workgroup owns ROWS consecutive victims (16, or fewer when that is needed to put a
// workgroup on every compute unit); its wavefronts split the n outranking
// candidates in 64-box tiles (lane = candidate c, victim r wave-uniform through scalar
// loads, exactly as in map_tile_kernel).  Each wavefront ends with one bit per victim,
// the workgroup ORs them through LDS and writes keep_out in input order.

// Which score compare decides "candidate c outranks victim r" for a whole tile:
// every candidate index below every victim index -> equal scores outrank (>=);
// every candidate index above -> strictly better only (>); the one tile that
// contains the victims themselves -> per lane.
enum { kGuardLowerIndex = 0, kGuardHigherIndex = 1, kGuardMixed = 2 };

// One victim row of the direct form: lane mask of the candidates that eliminate it.
template <bool FAST, int GUARD>
__device__ __forceinline__ unsigned long long direct_row(const float4 v, float v_score, int r, const float4 cb,
                                                         float c_score, float c_area, float c_T, int c,
                                                         const NmsThetaConst &th)
{
    bool hit;
    if (FAST)
        hit = nms_eliminates_fast(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, c_T);
    else
        hit = nms_eliminates_exact(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, c_area, th.theta);
    unsigned long long outranks;
    if (GUARD == kGuardLowerIndex) {
        outranks = __ballot(c_score >= v_score);
    } else if (GUARD == kGuardHigherIndex) {
        outranks = __ballot(c_score > v_score);
    } else {
        const unsigned long long lower = __ballot(c < r);
        outranks = (__ballot(c_score >= v_score) & lower) | (__ballot(c_score > v_score) & ~lower);
    }
    return __ballot(hit) & outranks;
}

template <bool FAST, int GUARD, bool CLAMP, int ROWS>
__device__ __forceinline__ unsigned direct_rows(const float4 *__restrict__ box4, const float *__restrict__ score,
                                                int v0, int n_f, const float4 cb, float c_score, float c_area, float c_T,
                                                int c, const NmsThetaConst &th)
{
    unsigned bits = 0;  // wave-uniform: bit k = victim v0+k is eliminated by a lane of this tile
    if (CLAMP) {
        // ragged last group of a frame: plain loop over the victims that exist
#pragma unroll 1
        for (int k = 0; k < ROWS && v0 + k < n_f; ++k) {
            const unsigned long long word = direct_row<FAST, GUARD>(box4[v0 + k], score[v0 + k], v0 + k, cb, c_score,
                                                                    c_area, c_T, c, th);
            bits |= (word != 0 ? 1u : 0u) << k;
        }
        return bits;
    }
    constexpr int kBatch = ROWS < 8 ? ROWS : 8;
#pragma unroll 1
    for (int half = 0; half < ROWS / kBatch; ++half) {
        // up to eight victims at a time: their scalar loads issue together, 40 SGPRs live
        float4 v[kBatch];
        float v_score[kBatch];
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            v[k] = box4[v0 + kBatch * half + k];
            v_score[k] = score[v0 + kBatch * half + k];
        }
        unsigned half_bits = 0;
#pragma unroll
        for (int k = 0; k < kBatch; ++k) {
            const unsigned long long word = direct_row<FAST, GUARD>(v[k], v_score[k], v0 + kBatch * half + k, cb,
                                                                    c_score, c_area, c_T, c, th);
            half_bits |= (word != 0 ? 1u : 0u) << k;
        }
        bits |= half_bits << (kBatch * half);
    }
    return bits;
}

template <bool FAST, bool CLAMP, int ROWS>
__device__ __forceinline__ unsigned direct_tile(const float4 *__restrict__ box4, const float *__restrict__ score,
                                                int v0, int n_f, int t, const float4 cb, float c_score, float c_area,
                                                float c_T, int c, const NmsThetaConst &th)
{
    if (t * kTile + kTile - 1 < v0)
        return direct_rows<FAST, kGuardLowerIndex, CLAMP, ROWS>(box4, score, v0, n_f, cb, c_score, c_area, c_T, c, th);
    if (t * kTile > v0 + ROWS - 1)
        return direct_rows<FAST, kGuardHigherIndex, CLAMP, ROWS>(box4, score, v0, n_f, cb, c_score, c_area, c_T, c, th);
    return direct_rows<FAST, kGuardMixed, CLAMP, ROWS>(box4, score, v0, n_f, cb, c_score, c_area, c_T, c, th);
}

template <bool FAST, int ROWS>
__global__ void __launch_bounds__(1024)
direct_kernel(const float *__restrict__ boxes, const float *__restrict__ scores, const int32_t *__restrict__ counts,
              int n_max, NmsThetaConst th, uint8_t *__restrict__ keep_out)
{
    __shared__ unsigned hits[16];
    const int f = blockIdx.y;
    const int v0 = blockIdx.x * ROWS;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n_waves = blockDim.x >> 6;
    const int n_f = frame_count(counts, f, n_max);
    uint8_t *keep_f = keep_out + (size_t)f * n_max;
    if (v0 >= n_f) {  // whole group beyond the frame's count (uniform for the workgroup)
        if (threadIdx.x < ROWS && v0 + (int)threadIdx.x < n_max) keep_f[v0 + threadIdx.x] = 0;
        return;
    }
    const float4 *box4 = reinterpret_cast<const float4 *>(boxes) + (size_t)f * n_max;
    const float *score = scores + (size_t)f * n_max;
    const int tiles = (n_f + kTile - 1) / kTile;
    const bool full = v0 + ROWS <= n_f;

    unsigned acc = 0;
    for (int t = wave; t < tiles; t += n_waves) {
        const int c = t * kTile + lane;
        const bool valid = c < n_f;
        const int cc = valid ? c : n_f - 1;
        const float4 cb = box4[cc];
        // a lane beyond the count never outranks anything: score -inf, index >= n_f
        const float c_score = valid ? score[cc] : -INFINITY;
        const float c_area = nms_box_area(cb.x, cb.y, cb.z, cb.w);
        const float c_T = FAST ? nms_pair_threshold(c_area, th.m) : 0.0f;
        if (full)
            acc |= direct_tile<FAST, false, ROWS>(box4, score, v0, n_f, t, cb, c_score, c_area, c_T, c, th);
        else
            acc |= direct_tile<FAST, true, ROWS>(box4, score, v0, n_f, t, cb, c_score, c_area, c_T, c, th);
    }
    if (lane == 0) hits[wave] = acc;
    __syncthreads();
    if (threadIdx.x < ROWS) {
        const int r = v0 + threadIdx.x;
        unsigned any = 0;
        for (int w = 0; w < n_waves; ++w) any |= hits[w];
        if (r < n_max) keep_f[r] = (r < n_f) ? (uint8_t)(((any >> threadIdx.x) & 1u) ^ 1u) : (uint8_t)0;
    }
}

// ----------------------------------------------------------------------------- reduce

// Lane = row.  Row tile tr owns tr + 1 words per row (the triangle), so a wavefront takes the
// tile rows p and T - 1 - p: T + 1 words of 512 contiguous bytes each, the same for every
// wavefront, all loads independent of each other (eight in flight per wavefront), no LDS and no
// barrier.  Each mask byte is read exactly once.  (Two rows per lane with 16-byte loads, and
// non-temporal loads, both measured slower.)
__global__ void __launch_bounds__(256)
reduce_rows_kernel(const unsigned long long *__restrict__ mask, const int32_t *__restrict__ order,
                   const int32_t *__restrict__ counts, int n_max, int n_pad, uint8_t *__restrict__ keep_out)
{
    const int f = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int T = n_pad / kTile;
    const int p = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * 4 + (threadIdx.x >> 6)));
    if (p >= (T + 1) / 2) return;
    const int n_f = frame_count(counts, f, n_max);
    const unsigned long long *m = mask + (size_t)f * ((size_t)T * n_pad);
    uint8_t *keep_f = keep_out + (size_t)f * n_max;
    const int32_t *order_f = order + (size_t)f * n_max;
#pragma unroll 1
    for (int half = 0; half < 2; ++half) {
        const int tr = half == 0 ? p : T - 1 - p;
        if (half == 1 && tr == p) break;  // odd T: the middle tile row has no partner
        const int row = tr * kTile + lane;
        unsigned long long acc = 0;
        if (tr * kTile < n_f) {  // tile rows beyond the count are not written by the map step
            const unsigned long long *col = m + row;
#pragma unroll 8
            for (int w = 0; w <= tr; ++w) acc |= col[(size_t)w * n_pad];
        }
        if (row < n_f)
            keep_f[order_f[row]] = (acc == 0) ? 1 : 0;
        else if (row < n_max)
            keep_f[row] = 0;  // input slots beyond the frame's count
    }
}

// ----------------------------------------------------------------------------- greedy sweep

// The classic sequential procedure on the same mask: rank r survives iff no SURVIVING
// better-ranked box eliminates it.  (Not what the paper's Algorithm 2 computes -- there
// every better-ranked box counts -- but the rule its introduction describes; offered as a
// selectable reduce.)  The state of the procedure lives in keep_out itself (0 = known dead).
//
// greedy_sweep_kernel settles one block of up to kSweepTiles tile rows (4096 ranks) per
// launch, one workgroup per frame walking the block's tile rows in rank order:
//   - the wavefront that owns tile t (t mod 4) settles its 64 rows: rows already marked
//     dead by earlier survivors are out; among the rest, survivors inside the tile are the
//     unique solution of  kept[r] = alive[r] and no kept c < r of this tile hits r,  found by
//     iterating that equation from kept = alive until it stops changing (row r is final
//     after r+1 rounds at most; typically a few rounds);
//   - after a barrier every wavefront applies tile t's survivors to the later tiles of the
//     block that it owns: dead |= (mask word of column tile t) & kept_t, one coalesced
//     512-byte read per tile, and records the result as a ballot in LDS (each tile has one
//     owner: no atomics).
// The mask words a step needs do not depend on the steps before it, only what is done with
// them does; they are fetched kSweepDepth steps ahead so that memory latency (about as long
// as four steps' work) stays off the dependent chain.
// Frames with more than one block alternate with greedy_apply_kernel, which applies a settled
// block's survivors to every later row in parallel.
// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// global load in flight, which would put the look-ahead fetches back on the dependent chain.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

constexpr int kSweepTiles = 64;
constexpr int kSweepDepth = 3;  // (depth + 1) x 17 loads must stay below the 63 that the hardware counter of outstanding loads can express
constexpr int kSweepOwned = kSweepTiles / 4;  // tiles of a block that one wavefront owns

struct SweepStage {
    unsigned long long later[kSweepOwned];  // column tile t: words of the later tiles this wavefront owns
    unsigned long long diag;                // column tile t, rows of tile t itself (owner only)
};

template <bool FIRST>
__global__ void __launch_bounds__(256)
greedy_sweep_kernel(const unsigned long long *__restrict__ mask, const int32_t *__restrict__ order,
                    const int32_t *__restrict__ counts, int n_max, int n_pad, int t0, uint8_t *__restrict__ keep_out)
{
    __shared__ unsigned long long kept_s[kSweepTiles];
    const int f = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n_f = frame_count(counts, f, n_max);
    const int tiles_f = (n_f + kTile - 1) / kTile;
    const int t1 = t0 + kSweepTiles < tiles_f ? t0 + kSweepTiles : tiles_f;  // this launch settles tiles t0 .. t1-1
    const unsigned long long *m = mask + (size_t)f * ((size_t)(n_pad / kTile) * n_pad);
    uint8_t *keep_f = keep_out + (size_t)f * n_max;
    const int32_t *order_f = order + (size_t)f * n_max;

    // A wavefront owns the tiles t0 + wave + 4i, i = 0..15 (t0 is a multiple of 4), and a lane
    // the row `lane` of each: bit i of my_dead / my_kept is the state of that row.  The first
    // block starts with every row alive, later blocks read what the apply kernel left in keep_out.
    unsigned my_dead = 0, my_kept = 0;
    // input index of this lane's row of each owned tile (-1: no such row); the loads are
    // independent of each other and issue together
    int my_index[kSweepOwned];
#pragma unroll
    for (int i = 0; i < kSweepOwned; ++i) {
        const int r = (t0 + wave + 4 * i) * kTile + lane;
        my_index[i] = (t0 + wave + 4 * i < t1 && r < n_f) ? order_f[r] : -1;
    }
    if (!FIRST) {
        uint8_t state[kSweepOwned];
#pragma unroll
        for (int i = 0; i < kSweepOwned; ++i) state[i] = my_index[i] >= 0 ? keep_f[my_index[i]] : (uint8_t)1;
#pragma unroll
        for (int i = 0; i < kSweepOwned; ++i) my_dead |= (state[i] == 0 ? 1u : 0u) << i;
    }

    // Every fetch issues the same 17 loads whatever t is (indices clamped into the block; words
    // fetched that way are never used) and the loop below holds no other global access: the
    // number of loads in flight is then known at compile time, and a step waits only for the
    // words it uses, not for the look-ahead behind them.
    auto fetch = [&](SweepStage &s, int t) {
        const int tt = t < t1 ? t : t1 - 1;
        int j = t + 1;
        j += (wave - j) & 3;  // first later tile owned by this wavefront
#pragma unroll
        for (int i = 0; i < kSweepOwned; ++i, j += 4) {
            const int jj = j < t1 ? j : t1 - 1;
            s.later[i] = m[(size_t)tt * n_pad + jj * kTile + lane];
        }
        s.diag = m[(size_t)tt * n_pad + tt * kTile + lane];
    };
    // One step: settle tile t with the words in `s`, apply its survivors, then reuse `s` for
    // the fetch of step t + kSweepDepth.  The stages are separate variables (s0, s1, s2 below),
    // not an indexed array, so each keeps its own registers while its loads are in flight.
    auto step = [&](SweepStage &s, int t) {
        if (t >= t1) return;  // uniform for the workgroup
        if (wave == (t & 3)) {
            const int i = (t - t0) >> 2;
            const bool alive = t * kTile + lane < n_f && ((my_dead >> i) & 1u) == 0;
            unsigned long long kept = __ballot(alive);
            for (int round = 0; round < kTile; ++round) {
                const unsigned long long next = __ballot(alive && (s.diag & kept) == 0);
                if (next == kept) break;
                kept = next;
            }
            if (lane == 0) kept_s[t - t0] = kept;
            my_kept |= (unsigned)((kept >> lane) & 1ull) << i;
        }
        lds_barrier();
        // survivors of tile t against this lane's rows of the later tiles the wavefront owns:
        // later[i] belongs to owned tile number first + i (numbers past the block are never read back)
        const unsigned long long kept_t = kept_s[t - t0];
        int j = t + 1;
        j += (wave - j) & 3;
        const int first = (j - t0) >> 2;
        unsigned hits = 0;
#pragma unroll
        for (int i = 0; i < kSweepOwned; ++i) hits |= ((s.later[i] & kept_t) != 0 ? 1u : 0u) << i;
        my_dead |= hits << first;
        fetch(s, t + kSweepDepth);
    };
    static_assert(kSweepDepth == 3, "the loop below is written out for three stages");
    if (t0 < t1) {
        SweepStage s0, s1, s2;
        fetch(s0, t0);
        fetch(s1, t0 + 1);
        fetch(s2, t0 + 2);
#pragma unroll 1
        for (int tb = t0; tb < t1; tb += kSweepDepth) {
            step(s0, tb);
            step(s1, tb + 1);
            step(s2, tb + 2);
        }
    }
#pragma unroll
    for (int i = 0; i < kSweepOwned; ++i)
        if (my_index[i] >= 0) keep_f[my_index[i]] = (uint8_t)((my_kept >> i) & 1u);
    if (FIRST)
        for (int i = n_f + (int)threadIdx.x; i < n_max; i += blockDim.x) keep_f[i] = 0;  // slots beyond the count
}

// Applies the survivors of the settled block of tile rows t0 .. t0+kSweepTiles-1 to every
// later row: a row with a surviving eliminator in the block is marked dead in keep_out.
// After the first block (FIRST) every later row is written, 1 = alive so far, which
// initialises the state.  One wavefront per later tile row, four per workgroup; the block's
// survivor words are rebuilt from keep_out into LDS by each workgroup.
template <bool FIRST>
__global__ void __launch_bounds__(256)
greedy_apply_kernel(const unsigned long long *__restrict__ mask, const int32_t *__restrict__ order,
                    const int32_t *__restrict__ counts, int n_max, int n_pad, int t0, uint8_t *__restrict__ keep_out)
{
    __shared__ unsigned long long kept_s[kSweepTiles];
    const int f = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n_f = frame_count(counts, f, n_max);
    const int first_row_tile = t0 + kSweepTiles + (int)blockIdx.x * 4;
    if (first_row_tile * kTile >= n_f) return;  // whole workgroup beyond the count (then the block below is full)
    uint8_t *keep_f = keep_out + (size_t)f * n_max;
    const int32_t *order_f = order + (size_t)f * n_max;
    for (int w = wave; w < kSweepTiles; w += 4) {
        const int r = (t0 + w) * kTile + lane;  // < n_f: a later tile row holds boxes, so the block is full
        const unsigned long long kept = __ballot(keep_f[order_f[r]] != 0);
        if (lane == 0) kept_s[w] = kept;
    }
    __syncthreads();
    const int j = first_row_tile + wave;
    const int row = j * kTile + lane;
    if (j * kTile >= n_f) return;
    const unsigned long long *col = mask + (size_t)f * ((size_t)(n_pad / kTile) * n_pad) + (size_t)t0 * n_pad + row;
    unsigned long long acc = 0;
#pragma unroll 8
    for (int w = 0; w < kSweepTiles; ++w) acc |= col[(size_t)w * n_pad] & kept_s[w];
    if (row < n_f) {
        if (FIRST)
            keep_f[order_f[row]] = acc != 0 ? 0 : 1;
        else if (acc != 0)
            keep_f[order_f[row]] = 0;
    }
}

// ----------------------------------------------------------------------------- greedy rule without a mask

// The classic sequential rule walked tile by tile in rank order, one workgroup (16
// wavefronts) per frame, no mask in memory.  Under this rule a box that is eliminated
// neither eliminates others nor needs any further test, so only the SURVIVORS are ever used
// as outranking boxes: about 600 of 4096 on frames like configuration 4, i.e. a seventh of
// the pair grid.  Worth it when a batch has about as many frames as the chip has compute
// units, since each frame is walked sequentially.
//
// A wavefront owns the tiles wave, wave + 16, wave + 32, wave + 48 and keeps their boxes in
// registers, lane = row; one wave-uniform 64-bit word per owned tile says which rows are
// eliminated (or do not exist).  For tile t = 0, 1, ...:
//   - its owner settles it: the rows still alive are visited in rank order; each one visited
//     is a survivor, is broadcast from its lane (v_readlane), eliminates the later rows of the
//     tile that it hits, and is appended to a list in LDS;
//   - barrier; every wavefront tests its later tiles against the list, one survivor at a
//     time (broadcast from the lane that read it from LDS), all 64 rows per instruction.
constexpr int kFusedWaves = 16;
constexpr int kFusedOwned = NMS_SORT_CHUNK / kTile / kFusedWaves;  // 4
constexpr long long kGreedyFusedBoxes = 128ll * 4096;  // nms_run_greedy_batched takes this route from frames * n_max boxes on

struct FusedCandidate {  // a survivor as an outranking box (fields a variant does not use are never read)
    float x1, y1, x2, y2, area, T, score;
    int label;
};

enum { kExTiesIgnore = 2, kExClasses = 4 };                       // flags of the variants (AUX)
enum { kExBoundary = 0, kExDivideGe = 1, kExDivideGt = 2 };      // how a variant decides the threshold (MODE)

// What the walk needs beyond the box table when it runs a variant of the rule (EX): see
// map_tile_ex_kernel below for the arithmetic.
struct FusedVariant {
    const float *ranked_score;    // [frames][n_pad], rank order (AUX)
    const int32_t *ranked_label;  // [frames][n_pad], rank order (AUX with labels)
    double boundary;              // rounding boundary of the division next to theta (MODE == kExBoundary)
    float offset;                 // 1 or 0
    int flags;
};

// Does candidate c eliminate the victim?  !EX: the default measure (MODE kExBoundary = the
// division-free form of nms_pair.h, else the literal division).  EX: the variants.
template <bool EX, bool IOU, int MODE, bool AUX>
__device__ __forceinline__ bool fused_hit(const float4 v, float v_area, float v_score, int v_label,
                                          const FusedCandidate &c, float theta, const FusedVariant &o)
{
    if (!EX) {
        if (MODE == kExBoundary) return nms_eliminates_fast(v.x, v.y, v.z, v.w, c.x1, c.y1, c.x2, c.y2, c.T);
        return nms_eliminates_exact(v.x, v.y, v.z, v.w, c.x1, c.y1, c.x2, c.y2, c.area, theta);
    }
    const float iw = fmaxf(0.0f, (fminf(v.z, c.x2) - fmaxf(v.x, c.x1)) + o.offset);
    const float ih = fmaxf(0.0f, (fminf(v.w, c.y2) - fmaxf(v.y, c.y1)) + o.offset);
    const float inter = iw * ih;
    const float denom = IOU ? (v_area + c.area) - inter : c.area;
    bool hit;
    if (MODE == kExBoundary && !IOU)
        hit = inter >= c.T;
    else if (MODE == kExBoundary)
        hit = (double)inter >= o.boundary * (double)denom;
    else if (MODE == kExDivideGe)
        hit = !(inter / denom < theta);
    else
        hit = inter / denom > theta;
    if (AUX) {
        hit = hit && ((o.flags & kExTiesIgnore) == 0 || c.score > v_score);
        hit = hit && ((o.flags & kExClasses) == 0 || c.label == v_label);
    }
    return hit;
}

// Lane `src` (wave-uniform) of a per-lane candidate, as a wave-uniform value.
__device__ __forceinline__ FusedCandidate broadcast_candidate(const FusedCandidate &mine, int src)
{
    FusedCandidate c;
    c.x1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine.x1), src));
    c.y1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine.y1), src));
    c.x2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine.x2), src));
    c.y2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine.y2), src));
    c.area = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine.area), src));
    c.T = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine.T), src));
    c.score = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, mine.score), src));
    c.label = __builtin_amdgcn_readlane(mine.label, src);
    return c;
}

template <bool EX, bool IOU, int MODE, bool AUX>
__global__ void __launch_bounds__(kFusedWaves * 64)
greedy_fused_kernel(const float *__restrict__ sorted5, const int32_t *__restrict__ order,
                    const int32_t *__restrict__ counts, int n_max, int n_pad, NmsThetaConst th, FusedVariant opt,
                    uint8_t *__restrict__ keep_out)
{
    __shared__ FusedCandidate list_s[2][kTile];  // survivors of tile t in buffer t & 1
    __shared__ int count_s[2];
    const int f = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n_f = frame_count(counts, f, n_max);
    const int tiles_f = (n_f + kTile - 1) / kTile;
    const float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    const float4 *box4 = reinterpret_cast<const float4 *>(sorted_f);
    const float *area = sorted_f + 4 * (size_t)n_pad;
    uint8_t *keep_f = keep_out + (size_t)f * n_max;
    const int32_t *order_f = order + (size_t)f * n_max;

    // the owned tiles: boxes (also in their role as outranking boxes) and the rows that are out
    float4 vb[kFusedOwned];
    FusedCandidate self[kFusedOwned];
    unsigned long long out[kFusedOwned];  // wave-uniform; bit r: row r is eliminated, settled or does not exist
#pragma unroll
    for (int i = 0; i < kFusedOwned; ++i) {
        const int tr = wave + kFusedWaves * i;
        const bool has = tr < tiles_f;
        const int r = has ? tr * kTile + lane : 0;  // rows of a partial last tile beyond n_f are padding rows of the table
        vb[i] = box4[r];
        FusedCandidate me;
        me.x1 = vb[i].x, me.y1 = vb[i].y, me.x2 = vb[i].z, me.y2 = vb[i].w;
        me.area = EX ? ((vb[i].z - vb[i].x) + opt.offset) * ((vb[i].w - vb[i].y) + opt.offset) : area[r];
        me.T = MODE == kExBoundary ? nms_pair_threshold(me.area, EX ? opt.boundary : th.m) : 0.0f;
        me.score = AUX ? opt.ranked_score[(size_t)f * n_pad + r] : 0.0f;
        me.label = (AUX && (opt.flags & kExClasses)) ? opt.ranked_label[(size_t)f * n_pad + r] : 0;
        self[i] = me;
        const int first = tr * kTile;
        out[i] = !has ? ~0ull : (first + kTile <= n_f ? 0ull : ~0ull << (n_f - first));
    }

    for (int t = 0; t < tiles_f; ++t) {
        const int buf = t & 1;
        if (wave == (t & (kFusedWaves - 1))) {
            // settle tile t = owned tile number t / 16
            float4 v = vb[0];
            FusedCandidate mine = self[0];
            unsigned long long todo = ~out[0];
#pragma unroll
            for (int i = 1; i < kFusedOwned; ++i) {
                if ((t >> 4) == i) {  // wave-uniform
                    v = vb[i];
                    mine = self[i];
                    todo = ~out[i];
                }
            }
            unsigned long long kept = 0;
            int count = 0;
            while (todo != 0) {
                const int c = (int)__builtin_ctzll(todo);  // best-ranked row still alive: a survivor
                todo &= todo - 1ull;
                kept |= 1ull << c;
                const FusedCandidate cand = broadcast_candidate(mine, c);
                const bool hit = fused_hit<EX, IOU, MODE, AUX>(v, mine.area, mine.score, mine.label, cand, th.theta, opt) &&
                                 lane > c;
                todo &= ~__ballot(hit);
                if (lane == 0) list_s[buf][count] = cand;
                ++count;
            }
            if (lane == 0) count_s[buf] = count;
            const int r = t * kTile + lane;
            if (r < n_f) keep_f[order_f[r]] = (uint8_t)((kept >> lane) & 1ull);
#pragma unroll
            for (int i = 0; i < kFusedOwned; ++i)
                if ((t >> 4) == i) out[i] = ~0ull;
        }
        lds_barrier();
        // the survivors of tile t against the later owned tiles that still have a row alive
        const int count = __builtin_amdgcn_readfirstlane(count_s[buf]);
        bool any = false;
#pragma unroll
        for (int i = 0; i < kFusedOwned; ++i) any = any || (wave + kFusedWaves * i > t && out[i] != ~0ull);
        if (count > 0 && any) {
            const FusedCandidate held = list_s[buf][lane < count ? lane : 0];  // lane k holds survivor k
            for (int k = 0; k < count; ++k) {
                const FusedCandidate cand = broadcast_candidate(held, k);
#pragma unroll
                for (int i = 0; i < kFusedOwned; ++i) {
                    if (wave + kFusedWaves * i > t && out[i] != ~0ull)  // wave-uniform
                        out[i] |= __ballot(fused_hit<EX, IOU, MODE, AUX>(vb[i], self[i].area, self[i].score, self[i].label,
                                                                          cand, th.theta, opt));
                }
            }
        }
    }
    for (int i = n_f + (int)threadIdx.x; i < n_max; i += blockDim.x) keep_f[i] = 0;  // slots beyond the count
}

// ----------------------------------------------------------------------------- map with options

// Rank-ordered scores and class labels (victims of a row are fetched with scalar loads, so
// the map kernel wants them contiguous in rank order like the box table).
__global__ void __launch_bounds__(256)
gather_ranked_kernel(const int32_t *__restrict__ order, const float *__restrict__ scores,
                     const int32_t *__restrict__ classes, const int32_t *__restrict__ counts, int n_max, int n_pad,
                     float *__restrict__ ranked_score, int32_t *__restrict__ ranked_class)
{
    const int f = blockIdx.y;
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    if (r >= n_pad) return;
    const int n_f = frame_count(counts, f, n_max);
    const bool real = r < n_f;
    const int idx = real ? order[(size_t)f * n_max + r] : 0;
    ranked_score[(size_t)f * n_pad + r] = real ? scores[(size_t)f * n_max + idx] : -INFINITY;
    if (classes != nullptr) ranked_class[(size_t)f * n_pad + r] = real ? classes[(size_t)f * n_max + idx] : 0;
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
template <bool IOU, int MODE, bool AUX>
__global__ void __launch_bounds__(kMapWaves * 64)
map_tile_ex_kernel(const float *__restrict__ sorted5, const float *__restrict__ ranked_score,
                   const int32_t *__restrict__ ranked_class, const int32_t *__restrict__ counts, int n_max, int n_pad,
                   int tiles, float theta, double boundary, float offset, int flags,
                   unsigned long long *__restrict__ mask)
{
    const int lane = threadIdx.x & 63;
    const int f = blockIdx.y;
    const int g = __builtin_amdgcn_readfirstlane((int)(blockIdx.x * kMapWaves + (threadIdx.x >> 6)));
    if (g >= tiles) return;
    const int n_f = frame_count(counts, f, n_max);
    int tr, tc;
    triangle_unit<1>(g, tr, tc);
    if (tr * kTile >= n_f) return;

    const float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    const float4 *box4 = reinterpret_cast<const float4 *>(sorted_f);
    const float *score_f = ranked_score + (size_t)f * n_pad;
    const int32_t *class_f = ranked_class + (size_t)f * n_pad;  // unwritten (but allocated) when no labels were given
    const bool ties_ignore = (flags & kExTiesIgnore) != 0;
    const bool labelled = (flags & kExClasses) != 0;

    const int c = tc * kTile + lane;
    const float4 cb = box4[c];
    const float c_area = ((cb.z - cb.x) + offset) * ((cb.w - cb.y) + offset);
    const float c_score = AUX ? score_f[c] : 0.0f;
    const int c_class = AUX ? class_f[c] : 0;
    const float c_T = (MODE == kExBoundary && !IOU) ? nms_pair_threshold(c_area, boundary) : 0.0f;

    const float4 *__restrict__ vb = box4 + tr * kTile;  // wave-uniform addresses: scalar loads
    const float *__restrict__ vs = score_f + tr * kTile;
    const int32_t *__restrict__ vc = class_f + tr * kTile;
    unsigned w_lo = 0, w_hi = 0;
    constexpr int kGroup = 8;
#pragma unroll 1
    for (int grp = 0; grp < kTile / kGroup; ++grp) {
        // a group's victims are fetched together, its words formed without a branch in between
        float4 v[kGroup];
        float v_score[kGroup];
        int v_class[kGroup];
#pragma unroll
        for (int k = 0; k < kGroup; ++k) {
            v[k] = vb[kGroup * grp + k];
            v_score[k] = AUX ? vs[kGroup * grp + k] : 0.0f;
            v_class[k] = AUX ? vc[kGroup * grp + k] : 0;
        }
        unsigned long long words[kGroup];
#pragma unroll
        for (int k = 0; k < kGroup; ++k) {
            const int r = kGroup * grp + k;
            const float iw = fmaxf(0.0f, (fminf(v[k].z, cb.z) - fmaxf(v[k].x, cb.x)) + offset);
            const float ih = fmaxf(0.0f, (fminf(v[k].w, cb.w) - fmaxf(v[k].y, cb.y)) + offset);
            const float inter = iw * ih;
            float denom = c_area;
            if (IOU) {
                const float v_area = ((v[k].z - v[k].x) + offset) * ((v[k].w - v[k].y) + offset);
                denom = (v_area + c_area) - inter;
            }
            bool hit;
            if (MODE == kExBoundary && !IOU)
                hit = inter >= c_T;  // the denominator is the lane's own area: one float32 threshold per box, as in nms_pair.h
            else if (MODE == kExBoundary)
                hit = (double)inter >= boundary * (double)denom;
            else if (MODE == kExDivideGe)
                hit = !(inter / denom < theta);
            else
                hit = inter / denom > theta;
            if (AUX) {
                hit = hit && (!ties_ignore || c_score > v_score[k]);
                hit = hit && (!labelled || c_class == v_class[k]);
            }
            unsigned long long word = __ballot(hit);
            if (tr == tc) word &= (1ull << r) - 1ull;  // only better-ranked boxes eliminate
            words[k] = word;
        }
#pragma unroll
        for (int k = 0; k < kGroup; ++k) {
            if (words[k] != 0) {  // wave-uniform
                const bool mine = (lane == kGroup * grp + k);
                w_lo = mine ? (unsigned)words[k] : w_lo;
                w_hi = mine ? (unsigned)(words[k] >> 32) : w_hi;
            }
        }
    }
    const int row = tr * kTile + lane;
    unsigned long long out = ((unsigned long long)w_hi << 32) | w_lo;
    if (row >= n_f) out = 0;
    mask[(size_t)f * ((size_t)(n_pad / kTile) * n_pad) + (size_t)tc * n_pad + row] = out;
}

// ----------------------------------------------------------------------------- the paper's matrix form

// Algorithm 1 with the paper's own data layout: the boolean matrix B as capacity x capacity
// bytes over the unsorted input, one element per ordered pair (i, j), the score guard
// evaluated per pair.  A wavefront owns 256 consecutive columns j (four per lane, kept in
// registers) and kMatRows consecutive rows i (wave-uniform, scalar loads); each lane stores
// its four bytes of a row as one 32-bit word, 256 contiguous bytes per wavefront and row.
// Every byte is written, so the paper's memset of B is not needed.
constexpr int kMatRows = 16;

template <bool FAST>
__global__ void __launch_bounds__(256)
map_matrix_kernel(const float *__restrict__ boxes, const float *__restrict__ scores, int n, int cap,
                  NmsThetaConst th, uint8_t *__restrict__ B)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int j0 = blockIdx.x * 256 + 4 * lane;
    const int i0 = (blockIdx.y * 4 + wave) * kMatRows;
    if (i0 >= cap) return;
    const float4 *box4 = reinterpret_cast<const float4 *>(boxes);

    float4 cb[4];
    float c_score[4], c_area[4], c_T[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int c = j0 + q;
        const bool valid = c < n;
        cb[q] = valid ? box4[c] : make_float4(0.f, 0.f, 0.f, 0.f);
        c_score[q] = valid ? scores[c] : -INFINITY;  // an unused slot never outranks anything
        c_area[q] = nms_box_area(cb[q].x, cb[q].y, cb[q].z, cb[q].w);
        c_T[q] = FAST ? nms_pair_threshold(c_area[q], th.m) : 0.0f;
    }

    const int i_end = i0 + kMatRows < cap ? i0 + kMatRows : cap;
    for (int i = i0; i < i_end; ++i) {
        unsigned word = 0x01010101u;  // rows of unused slots: never guarded, stay 1
        if (i < n) {
            const float4 v = box4[i];
            const float v_score = scores[i];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                bool hit;
                if (FAST)
                    hit = nms_eliminates_fast(v.x, v.y, v.z, v.w, cb[q].x, cb[q].y, cb[q].z, cb[q].w, c_T[q]);
                else
                    hit = nms_eliminates_exact(v.x, v.y, v.z, v.w, cb[q].x, cb[q].y, cb[q].z, cb[q].w, c_area[q],
                                               th.theta);
                const bool outranks = c_score[q] > v_score || (c_score[q] == v_score && j0 + q < i);
                if (hit && outranks) word &= ~(1u << (8 * q));
            }
        }
        if (j0 < cap) *reinterpret_cast<unsigned *>(B + (size_t)i * cap + j0) = word;
    }
}

// Algorithm 2 as printed: one workgroup per row i with capacity / k threads; thread t
// looks at column t of each of the k partitions in turn, and a block-wide AND
// (__syncthreads_and: barrier plus wave ballots combined through LDS; CDNA has no barrier
// instruction that reduces) folds each partition into V_i.
__global__ void __launch_bounds__(1024)
reduce_matrix_kernel(const uint8_t *__restrict__ B, int cap, int k, uint8_t *__restrict__ V)
{
    const int i = blockIdx.x;
    const int part = cap / k;  // == blockDim.x
    size_t j = (size_t)i * cap + threadIdx.x;
    int v = __syncthreads_and(B[j]);
    for (int p = 1; p < k; ++p) {
        j += part;
        v = __syncthreads_and(v && B[j]);
    }
    if (threadIdx.x == 0) V[i] = (uint8_t)(v ? 1 : 0);
}

// ----------------------------------------------------------------------------- host side

struct Pool {
    void *ws = nullptr;
    size_t bytes = 0;
    int n_max = 0;
    int frames_max = 0;
};
Pool g_pool;

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

inline bool sizes_ok(int n_max, int frames, int *status)
{
    if (n_max < 0 || frames < 0) { *status = NMS_ERR_INVALID_ARG; return false; }
    if (n_max > NMS_MAX_N || frames > NMS_MAX_FRAMES) { *status = NMS_ERR_TOO_LARGE; return false; }
    return true;
}

inline bool is_nan(float v)
{
    uint32_t b;
    memcpy(&b, &v, sizeof b);
    return (b & 0x7fffffffu) > 0x7f800000u;
}

thread_local hipError_t g_last_hip_error = hipSuccess;

// The runtime's "last error" is per thread and sticky across libraries: an unrelated
// earlier failure (for example a probe made by the host framework) would otherwise be
// reported as ours.  begin_launch() discards it, launch_status() reads ours.
inline void begin_launch() { (void)hipGetLastError(); }

inline int launch_status()
{
    const hipError_t e = hipGetLastError();
    if (e == hipSuccess) return NMS_OK;
    g_last_hip_error = e;
    return NMS_ERR_LAUNCH;
}

int rank_launch(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                int32_t *order, float *sorted5, void *workspace, uint8_t *keep_preset, float4 *ysc, unsigned *ytile,
                hipStream_t stream)
{
    const int n_pad = nms_padded_n(n_max);
    const int n_chunks = (n_max + kChunk - 1) / kChunk;
    int threads = 64;  // four keys per thread, at least one wavefront
    const int widest = n_max < kChunk ? n_max : kChunk;
    while (threads < 1024 && threads * 4 < widest) threads <<= 1;
    auto *keys_ws = static_cast<unsigned long long *>(workspace);
    begin_launch();
    rank_chunk_kernel<<<dim3(n_chunks, frames), dim3(threads), 0, stream>>>(
        boxes, scores, counts, n_max, n_pad, n_chunks, order, sorted5, keys_ws, keep_preset, ysc, ytile);
    int st = launch_status();
    if (st != NMS_OK || n_chunks == 1) return st;
    begin_launch();
    rank_merge_kernel<<<dim3((n_pad + 255) / 256, frames), dim3(256), 0, stream>>>(
        boxes, counts, n_max, n_pad, n_chunks, keys_ws, order, sorted5, ysc, ytile);
    return launch_status();
}

// Frames small enough that launch latency, not arithmetic, decides: one launch of the
// direct form instead of rank + map.  (Twice the pairs and two more compares per pair:
// about 2.5x the VALU work of the ranked triangle.)
inline bool use_direct_form(int n_max, int frames)
{
    return n_max <= 4096 && (long long)frames * n_max * n_max <= (1ll << 25);
}

int direct_launch(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                  float threshold, uint8_t *keep_out, hipStream_t stream)
{
    const NmsThetaConst th = nms_make_theta_const(threshold);
    const int tiles = (n_max + kTile - 1) / kTile;
    const int waves = tiles < 16 ? tiles : 16;
    // victims per workgroup: 16, or 8 / 4 when that is what it takes to have a workgroup for
    // every compute unit (a single 1024-box frame is 64 workgroups of 16 rows on a 256-CU chip)
    int rows = 16;
    while (rows > 4 && (long long)frames * ((n_max + rows - 1) / rows) < 256) rows >>= 1;
    const dim3 grid((n_max + rows - 1) / rows, frames);
    begin_launch();
#define NMS_LAUNCH_DIRECT(FAST_, ROWS_) \
    direct_kernel<FAST_, ROWS_><<<grid, dim3(waves * 64), 0, stream>>>(boxes, scores, counts, n_max, th, keep_out)
    if (th.fast) {
        if (rows == 16) NMS_LAUNCH_DIRECT(true, 16); else if (rows == 8) NMS_LAUNCH_DIRECT(true, 8); else NMS_LAUNCH_DIRECT(true, 4);
    } else {
        if (rows == 16) NMS_LAUNCH_DIRECT(false, 16); else if (rows == 8) NMS_LAUNCH_DIRECT(false, 8); else NMS_LAUNCH_DIRECT(false, 4);
    }
#undef NMS_LAUNCH_DIRECT
    return launch_status();
}

template <bool WRITE_MASK>
int map_launch(const float *sorted5, const int32_t *counts, int n_max, int frames, float threshold,
               unsigned long long *mask, const int32_t *order, uint8_t *keep_out, const float4 *ysc,
               const unsigned *ytile, hipStream_t stream)
{
    const int n_pad = nms_padded_n(n_max);
    const int T = n_pad / kTile;
    // four tiles per wavefront when that still leaves every SIMD several wavefronts
    const bool super4 = (long long)frames * triangle_units(T, 4) >= 16384;
    const int tiles = triangle_units(T, super4 ? 4 : 1);  // work units, one per wavefront
    const NmsThetaConst th = nms_make_theta_const(threshold);
    const int tile_blocks = (tiles + kMapWaves - 1) / kMapWaves;
    // batches: one frame per XCD at a time (see the kernel); a few large frames: spread each over all XCDs
    const int xcd_frames = frames >= 8 ? 1 : 0;
    const dim3 grid = xcd_frames ? dim3((unsigned)(((frames + 7) / 8) * 8 * tile_blocks)) : dim3(tile_blocks, frames);
    const dim3 block(kMapWaves * 64);
    begin_launch();
#define NMS_LAUNCH_MAP(FAST_, SUPER_)                                                                             \
    map_tile_kernel<FAST_, WRITE_MASK, SUPER_><<<grid, block, 0, stream>>>(sorted5, counts, n_max, n_pad, tiles,  \
                                                                           tile_blocks, frames, xcd_frames, th,   \
                                                                           mask, order, keep_out, ysc, ytile)
    if (th.fast) {
        if (super4) NMS_LAUNCH_MAP(true, 4); else NMS_LAUNCH_MAP(true, 1);
    } else {
        if (super4) NMS_LAUNCH_MAP(false, 4); else NMS_LAUNCH_MAP(false, 1);
    }
#undef NMS_LAUNCH_MAP
    return launch_status();
}

}  // namespace

// ----------------------------------------------------------------------------- C ABI

extern "C" {

const char *nms_status_string(int status)
{
    switch (status) {
    case NMS_OK: return "ok";
    case NMS_ERR_INVALID_ARG: return "invalid argument";
    case NMS_ERR_TOO_LARGE: return "size beyond NMS_MAX_N or NMS_MAX_FRAMES";
    case NMS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case NMS_ERR_LAUNCH: return "kernel launch failed";
    default: return "unknown status";
    }
}

int nms_version(void) { return NMS_VERSION; }

const char *nms_last_launch_error(void) { return hipGetErrorString(g_last_hip_error); }

int nms_padded_n(int n)
{
    if (n < 0 || n > NMS_MAX_N) return 0;
    return (n + kTile - 1) / kTile * kTile;
}

size_t nms_mask_words(int n)
{
    if (n < 0 || n > NMS_MAX_N) return 0;
    const size_t n_pad = (size_t)nms_padded_n(n);
    return (n_pad / kTile) * n_pad;
}

size_t nms_sort_workspace_bytes(int n_max, int frames)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return 0;
    if (n_max <= kChunk) return 0;
    return align256((size_t)frames * nms_padded_n(n_max) * sizeof(unsigned long long));
}

size_t nms_workspace_bytes(int n_max, int frames)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return 0;
    const size_t n_pad = (size_t)nms_padded_n(n_max);
    return align256((size_t)frames * n_max * sizeof(int32_t))               // order
         + align256((size_t)frames * 5 * n_pad * sizeof(float))             // sorted5
         + align256((size_t)frames * n_pad * 4 * sizeof(float))             // y-scaled boxes
         + align256((size_t)frames * (n_pad / kTile) * sizeof(unsigned))    // tile flags
         + nms_sort_workspace_bytes(n_max, frames);                         // chunk keys
}

int nms_sort_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                     int32_t *order, float *sorted5, void *workspace, size_t ws_bytes, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!boxes || !scores || !order || !sorted5) return NMS_ERR_INVALID_ARG;
    const size_t need = nms_sort_workspace_bytes(n_max, frames);
    if (need != 0 && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255))) return NMS_ERR_WORKSPACE;
    return rank_launch(boxes, scores, counts, n_max, frames, order, sorted5, workspace, nullptr, nullptr, nullptr,
                       static_cast<hipStream_t>(stream));
}

int nms_sort(const float *boxes, const float *scores, int n, int32_t *order, float *sorted5,
             void *workspace, size_t ws_bytes, void *stream)
{
    return nms_sort_batched(boxes, scores, nullptr, n, 1, order, sorted5, workspace, ws_bytes, stream);
}

int nms_overlap_mask_batched(const float *sorted5, const int32_t *counts, int n_max, int frames,
                             float threshold, uint64_t *mask, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!sorted5 || !mask) return NMS_ERR_INVALID_ARG;
    return map_launch<true>(sorted5, counts, n_max, frames, threshold,
                            reinterpret_cast<unsigned long long *>(mask), nullptr, nullptr, nullptr, nullptr,
                            static_cast<hipStream_t>(stream));
}

int nms_overlap_mask(const float *sorted5, int n, float threshold, uint64_t *mask, void *stream)
{
    return nms_overlap_mask_batched(sorted5, nullptr, n, 1, threshold, mask, stream);
}

int nms_reduce_batched(const uint64_t *mask, const int32_t *order, const int32_t *counts, int n_max, int frames,
                       uint8_t *keep_out, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!mask || !order || !keep_out) return NMS_ERR_INVALID_ARG;
    const int n_pad = nms_padded_n(n_max);
    begin_launch();
    const int row_pairs = (n_pad / kTile + 1) / 2;  // one wavefront per pair of tile rows, four per workgroup
    reduce_rows_kernel<<<dim3((row_pairs + 3) / 4, frames), dim3(256), 0, static_cast<hipStream_t>(stream)>>>(
        reinterpret_cast<const unsigned long long *>(mask), order, counts, n_max, n_pad, keep_out);
    return launch_status();
}

int nms_reduce(const uint64_t *mask, const int32_t *order, int n, uint8_t *keep_out, void *stream)
{
    return nms_reduce_batched(mask, order, nullptr, n, 1, keep_out, stream);
}

// Carve-up of the fused path's workspace (every part 256-byte aligned).
struct RunWorkspace {
    int32_t *order;     // [frames][n_max]
    float *sorted5;     // [frames][5 * n_pad]
    float4 *ysc;        // [frames][n_pad]       boxes with y * NMS_YSCALE, rank order
    unsigned *ytile;    // [frames][n_pad / 64]  1 = every box of the tile may use the y-scaled form
    void *keys;         // rank scratch (n_max > NMS_SORT_CHUNK only)
    char *end;
};

inline RunWorkspace carve_workspace(void *workspace, int n_max, int frames)
{
    const size_t n_pad = (size_t)nms_padded_n(n_max);
    RunWorkspace w;
    char *p = static_cast<char *>(workspace);
    w.order = reinterpret_cast<int32_t *>(p);
    p += align256((size_t)frames * n_max * sizeof(int32_t));
    w.sorted5 = reinterpret_cast<float *>(p);
    p += align256((size_t)frames * 5 * n_pad * sizeof(float));
    w.ysc = reinterpret_cast<float4 *>(p);
    p += align256((size_t)frames * n_pad * sizeof(float4));
    w.ytile = reinterpret_cast<unsigned *>(p);
    p += align256((size_t)frames * (n_pad / kTile) * sizeof(unsigned));
    w.keys = p;
    p += nms_sort_workspace_bytes(n_max, frames);
    w.end = p;
    return w;
}

enum Route { kRouteAuto = 0, kRouteRanked = 1, kRouteDirect = 2 };

static int run_routed(Route route, const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                      float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream,
                      void *const *events)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!boxes || !scores || !keep_out) return NMS_ERR_INVALID_ARG;
    const bool direct = route == kRouteDirect || (route == kRouteAuto && use_direct_form(n_max, frames));
    if (route != kRouteDirect) {  // the automatic route validates the workspace whichever way it goes
        const size_t need = nms_workspace_bytes(n_max, frames);
        if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255)) return NMS_ERR_WORKSPACE;
    }

    hipStream_t s = static_cast<hipStream_t>(stream);
    auto mark = [&](int i) {
        if (!events || !events[i]) return true;
        const hipError_t e = hipEventRecord(static_cast<hipEvent_t>(events[i]), s);
        if (e != hipSuccess) g_last_hip_error = e;
        return e == hipSuccess;
    };
    if (!mark(0)) return NMS_ERR_LAUNCH;
    if (direct) {
        if (!mark(1)) return NMS_ERR_LAUNCH;  // no rank step on this route
        st = direct_launch(boxes, scores, counts, n_max, frames, threshold, keep_out, s);
        if (st != NMS_OK) return st;
        return mark(2) ? NMS_OK : NMS_ERR_LAUNCH;
    }

    const RunWorkspace w = carve_workspace(workspace, n_max, frames);
    st = rank_launch(boxes, scores, counts, n_max, frames, w.order, w.sorted5, w.keys, keep_out, w.ysc, w.ytile, s);
    if (st != NMS_OK) return st;
    if (!mark(1)) return NMS_ERR_LAUNCH;
    st = map_launch<false>(w.sorted5, counts, n_max, frames, threshold, nullptr, w.order, keep_out, w.ysc, w.ytile, s);
    if (st != NMS_OK) return st;
    return mark(2) ? NMS_OK : NMS_ERR_LAUNCH;
}

int nms_run_batched_profiled(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                             float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream,
                             void *const *events)
{
    return run_routed(kRouteAuto, boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, ws_bytes,
                      stream, events);
}

int nms_run_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                    float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream)
{
    return run_routed(kRouteAuto, boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, ws_bytes,
                      stream, nullptr);
}

int nms_run_ranked_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                           float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream)
{
    return run_routed(kRouteRanked, boxes, scores, counts, n_max, frames, threshold, keep_out, workspace, ws_bytes,
                      stream, nullptr);
}

int nms_run_direct_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                           float threshold, uint8_t *keep_out, void *stream)
{
    return run_routed(kRouteDirect, boxes, scores, counts, n_max, frames, threshold, keep_out, nullptr, 0, stream,
                      nullptr);
}

int nms_reduce_greedy_batched(const uint64_t *mask, const int32_t *order, const int32_t *counts, int n_max,
                              int frames, uint8_t *keep_out, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!mask || !order || !keep_out) return NMS_ERR_INVALID_ARG;
    const int n_pad = nms_padded_n(n_max);
    const int T = n_pad / kTile;
    const unsigned long long *m = reinterpret_cast<const unsigned long long *>(mask);
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (int t0 = 0; t0 < T; t0 += kSweepTiles) {
        begin_launch();
        if (t0 == 0)
            greedy_sweep_kernel<true><<<dim3(frames), dim3(256), 0, s>>>(m, order, counts, n_max, n_pad, t0, keep_out);
        else
            greedy_sweep_kernel<false><<<dim3(frames), dim3(256), 0, s>>>(m, order, counts, n_max, n_pad, t0, keep_out);
        st = launch_status();
        if (st != NMS_OK) return st;
        const int later = T - (t0 + kSweepTiles);  // tile rows after this block
        if (later <= 0) break;
        const dim3 grid((later + 3) / 4, frames);
        begin_launch();
        if (t0 == 0)
            greedy_apply_kernel<true><<<grid, dim3(256), 0, s>>>(m, order, counts, n_max, n_pad, t0, keep_out);
        else
            greedy_apply_kernel<false><<<grid, dim3(256), 0, s>>>(m, order, counts, n_max, n_pad, t0, keep_out);
        st = launch_status();
        if (st != NMS_OK) return st;
    }
    return NMS_OK;
}

int nms_reduce_greedy(const uint64_t *mask, const int32_t *order, int n, uint8_t *keep_out, void *stream)
{
    return nms_reduce_greedy_batched(mask, order, nullptr, n, 1, keep_out, stream);
}

size_t nms_greedy_workspace_bytes(int n_max, int frames)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return 0;
    return nms_workspace_bytes(n_max, frames) + align256((size_t)frames * nms_mask_words(n_max) * sizeof(uint64_t));
}

// rank, then greedy_fused_kernel (frames of at most NMS_SORT_CHUNK boxes)
static int run_greedy_fused(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                            float threshold, uint8_t *keep_out, void *workspace, hipStream_t s)
{
    const RunWorkspace w = carve_workspace(workspace, n_max, frames);
    int st = rank_launch(boxes, scores, counts, n_max, frames, w.order, w.sorted5, w.keys, nullptr, nullptr, nullptr, s);
    if (st != NMS_OK) return st;
    const NmsThetaConst th = nms_make_theta_const(threshold);
    const int n_pad = nms_padded_n(n_max);
    begin_launch();
    const FusedVariant none = {nullptr, nullptr, 0.0, 1.0f, 0};
    if (th.fast)
        greedy_fused_kernel<false, false, kExBoundary, false><<<dim3(frames), dim3(kFusedWaves * 64), 0, s>>>(
            w.sorted5, w.order, counts, n_max, n_pad, th, none, keep_out);
    else
        greedy_fused_kernel<false, false, kExDivideGe, false><<<dim3(frames), dim3(kFusedWaves * 64), 0, s>>>(
            w.sorted5, w.order, counts, n_max, n_pad, th, none, keep_out);
    return launch_status();
}

int nms_run_greedy_fused_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                                 float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (n_max > kChunk) return NMS_ERR_TOO_LARGE;
    if (is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!boxes || !scores || !keep_out) return NMS_ERR_INVALID_ARG;
    if (!workspace || ws_bytes < nms_workspace_bytes(n_max, frames) || ((uintptr_t)workspace & 255))
        return NMS_ERR_WORKSPACE;
    return run_greedy_fused(boxes, scores, counts, n_max, frames, threshold, keep_out, workspace,
                            static_cast<hipStream_t>(stream));
}

int nms_run_greedy_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                           float threshold, uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!boxes || !scores || !keep_out) return NMS_ERR_INVALID_ARG;
    if (!workspace || ws_bytes < nms_greedy_workspace_bytes(n_max, frames) || ((uintptr_t)workspace & 255))
        return NMS_ERR_WORKSPACE;
    // batches with a frame for (nearly) every compute unit: one workgroup walks each frame, no mask
    // (measured crossover against rank + mask + sweep: 128 frames of 4096 boxes, 256 of 2048)
    if (n_max <= kChunk && (long long)frames * n_max >= kGreedyFusedBoxes)
        return run_greedy_fused(boxes, scores, counts, n_max, frames, threshold, keep_out, workspace,
                                static_cast<hipStream_t>(stream));
    const RunWorkspace w = carve_workspace(workspace, n_max, frames);
    unsigned long long *mask = reinterpret_cast<unsigned long long *>(w.end);
    int32_t *order = w.order;

    hipStream_t s = static_cast<hipStream_t>(stream);
    st = rank_launch(boxes, scores, counts, n_max, frames, w.order, w.sorted5, w.keys, nullptr, w.ysc, w.ytile, s);
    if (st != NMS_OK) return st;
    st = map_launch<true>(w.sorted5, counts, n_max, frames, threshold, mask, nullptr, nullptr, w.ysc, w.ytile, s);
    if (st != NMS_OK) return st;
    return nms_reduce_greedy_batched(reinterpret_cast<const uint64_t *>(mask), order, counts, n_max, frames, keep_out,
                                     stream);
}

size_t nms_ex_workspace_bytes(int n_max, int frames)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return 0;
    return nms_greedy_workspace_bytes(n_max, frames)
         + 2 * align256((size_t)frames * nms_padded_n(n_max) * sizeof(float));  // ranked scores, ranked labels
}

int nms_run_ex_batched(const float *boxes, const float *scores, const int32_t *counts, int n_max, int frames,
                       float threshold, const nms_options *options, uint8_t *keep_out,
                       void *workspace, size_t ws_bytes, void *stream)
{
    int st;
    if (!sizes_ok(n_max, frames, &st)) return st;
    if (is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    nms_options opt = {NMS_RULE_PAPER, NMS_MEASURE_OUTRANKING_AREA, NMS_COMPARE_GE, NMS_TIES_BY_INDEX, 1.0f, 0, nullptr};
    if (options) opt = *options;
    if ((opt.rule | opt.measure | opt.compare | opt.ties) & ~1) return NMS_ERR_INVALID_ARG;
    if (opt.reserved != 0 || !(opt.pixel_offset == 0.0f || opt.pixel_offset == 1.0f)) return NMS_ERR_INVALID_ARG;
    if (n_max == 0 || frames == 0) return NMS_OK;
    if (!boxes || !scores || !keep_out) return NMS_ERR_INVALID_ARG;
    if (!workspace || ws_bytes < nms_ex_workspace_bytes(n_max, frames) || ((uintptr_t)workspace & 255))
        return NMS_ERR_WORKSPACE;

    const int n_pad = nms_padded_n(n_max);
    const RunWorkspace w = carve_workspace(workspace, n_max, frames);
    char *p = w.end;
    unsigned long long *mask = reinterpret_cast<unsigned long long *>(p);
    p += align256((size_t)frames * nms_mask_words(n_max) * sizeof(uint64_t));
    float *ranked_score = reinterpret_cast<float *>(p);
    p += align256((size_t)frames * n_pad * sizeof(float));
    int32_t *ranked_class = reinterpret_cast<int32_t *>(p);

    hipStream_t s = static_cast<hipStream_t>(stream);
    st = rank_launch(boxes, scores, counts, n_max, frames, w.order, w.sorted5, w.keys, nullptr, nullptr, nullptr, s);
    if (st != NMS_OK) return st;
    begin_launch();
    gather_ranked_kernel<<<dim3((n_pad + 255) / 256, frames), dim3(256), 0, s>>>(
        w.order, scores, opt.classes, counts, n_max, n_pad, ranked_score, ranked_class);
    st = launch_status();
    if (st != NMS_OK) return st;

    const int tiles = triangle_units(n_pad / kTile, 1);
    const dim3 grid((tiles + kMapWaves - 1) / kMapWaves, frames);
    // rounding boundary of the division next to theta, exact in float64: below theta for ">=", above it for ">"
    double boundary = 0.0;
    bool divide = true;
    if (threshold >= 0x1p-40f && threshold <= 0x1p20f) {
        uint32_t bits;
        memcpy(&bits, &threshold, sizeof bits);
        const uint32_t other_bits = opt.compare == NMS_COMPARE_GT ? bits + 1u : bits - 1u;
        float other;
        memcpy(&other, &other_bits, sizeof other);
        boundary = 0.5 * ((double)threshold + (double)other);
        divide = false;
    }
    const int flags = (opt.ties == NMS_TIES_IGNORE ? kExTiesIgnore : 0) | (opt.classes ? kExClasses : 0);
    const int mode = !divide ? kExBoundary : (opt.compare == NMS_COMPARE_GT ? kExDivideGt : kExDivideGe);
    const bool iou = opt.measure == NMS_MEASURE_IOU;
    const bool aux = flags != 0;
    if (opt.rule == NMS_RULE_GREEDY && n_max <= kChunk && (long long)frames * n_max >= kGreedyFusedBoxes) {
        // large batches under the greedy rule: the mask-free walk, one workgroup per frame
        const NmsThetaConst th = nms_make_theta_const(threshold);
        const FusedVariant v = {ranked_score, ranked_class, boundary, opt.pixel_offset, flags};
        begin_launch();
#define NMS_LAUNCH_WALK(IOU_, MODE_, AUX_)                                                          \
    greedy_fused_kernel<true, IOU_, MODE_, AUX_><<<dim3(frames), dim3(kFusedWaves * 64), 0, s>>>(   \
        w.sorted5, w.order, counts, n_max, n_pad, th, v, keep_out)
#define NMS_LAUNCH_WALK_MODE(IOU_, AUX_)                                                  \
    do {                                                                                  \
        if (mode == kExBoundary) NMS_LAUNCH_WALK(IOU_, kExBoundary, AUX_);                \
        else if (mode == kExDivideGe) NMS_LAUNCH_WALK(IOU_, kExDivideGe, AUX_);           \
        else NMS_LAUNCH_WALK(IOU_, kExDivideGt, AUX_);                                    \
    } while (0)
        if (iou) {
            if (aux) NMS_LAUNCH_WALK_MODE(true, true); else NMS_LAUNCH_WALK_MODE(true, false);
        } else {
            if (aux) NMS_LAUNCH_WALK_MODE(false, true); else NMS_LAUNCH_WALK_MODE(false, false);
        }
#undef NMS_LAUNCH_WALK_MODE
#undef NMS_LAUNCH_WALK
        return launch_status();
    }
    begin_launch();
#define NMS_LAUNCH_EX(IOU_, MODE_, AUX_)                                                                          \
    map_tile_ex_kernel<IOU_, MODE_, AUX_><<<grid, dim3(kMapWaves * 64), 0, s>>>(                                 \
        w.sorted5, ranked_score, ranked_class, counts, n_max, n_pad, tiles, threshold, boundary, opt.pixel_offset, \
        flags, mask)
#define NMS_LAUNCH_EX_MODE(IOU_, AUX_)                                                    \
    do {                                                                                  \
        if (mode == kExBoundary) NMS_LAUNCH_EX(IOU_, kExBoundary, AUX_);                  \
        else if (mode == kExDivideGe) NMS_LAUNCH_EX(IOU_, kExDivideGe, AUX_);             \
        else NMS_LAUNCH_EX(IOU_, kExDivideGt, AUX_);                                      \
    } while (0)
    if (iou) {
        if (aux) NMS_LAUNCH_EX_MODE(true, true); else NMS_LAUNCH_EX_MODE(true, false);
    } else {
        if (aux) NMS_LAUNCH_EX_MODE(false, true); else NMS_LAUNCH_EX_MODE(false, false);
    }
#undef NMS_LAUNCH_EX_MODE
#undef NMS_LAUNCH_EX
    st = launch_status();
    if (st != NMS_OK) return st;
    if (opt.rule == NMS_RULE_GREEDY)
        return nms_reduce_greedy_batched(reinterpret_cast<const uint64_t *>(mask), w.order, counts, n_max, frames,
                                         keep_out, stream);
    return nms_reduce_batched(reinterpret_cast<const uint64_t *>(mask), w.order, counts, n_max, frames, keep_out,
                              stream);
}

int nms_map_matrix(const float *boxes, const float *scores, int n, int capacity, float threshold,
                   uint8_t *B, void *stream)
{
    if (n < 0 || capacity < 0) return NMS_ERR_INVALID_ARG;
    if (capacity > NMS_MAX_MATRIX) return NMS_ERR_TOO_LARGE;
    if (n > capacity || capacity % kTile != 0 || is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    if (capacity == 0) return NMS_OK;
    if (!B || (n > 0 && (!boxes || !scores))) return NMS_ERR_INVALID_ARG;
    const NmsThetaConst th = nms_make_theta_const(threshold);
    const dim3 grid((capacity + 255) / 256, (capacity + 4 * kMatRows - 1) / (4 * kMatRows));
    hipStream_t s = static_cast<hipStream_t>(stream);
    begin_launch();
    if (th.fast)
        map_matrix_kernel<true><<<grid, dim3(256), 0, s>>>(boxes, scores, n, capacity, th, B);
    else
        map_matrix_kernel<false><<<grid, dim3(256), 0, s>>>(boxes, scores, n, capacity, th, B);
    return launch_status();
}

int nms_reduce_matrix(const uint8_t *B, int capacity, int k, uint8_t *V, void *stream)
{
    if (capacity < 0 || k < 1) return NMS_ERR_INVALID_ARG;
    if (capacity > NMS_MAX_MATRIX) return NMS_ERR_TOO_LARGE;
    if (capacity % kTile != 0) return NMS_ERR_INVALID_ARG;
    if (capacity == 0) return NMS_OK;
    if (capacity % k != 0 || capacity / k > 1024 || !B || !V) return NMS_ERR_INVALID_ARG;
    begin_launch();
    reduce_matrix_kernel<<<dim3(capacity), dim3(capacity / k), 0, static_cast<hipStream_t>(stream)>>>(B, capacity, k, V);
    return launch_status();
}

int nms_run_ws(const float *boxes, const float *scores, int n, float threshold,
               uint8_t *keep_out, void *workspace, size_t ws_bytes, void *stream)
{
    return nms_run_batched(boxes, scores, nullptr, n, 1, threshold, keep_out, workspace, ws_bytes, stream);
}

int nms_init(int n_max, int frames_max, void *workspace, size_t ws_bytes)
{
    int st;
    if (!sizes_ok(n_max, frames_max, &st)) return st;
    if (n_max == 0 || frames_max == 0) return NMS_ERR_INVALID_ARG;
    if (!workspace || ((uintptr_t)workspace & 255) || ws_bytes < nms_workspace_bytes(n_max, frames_max))
        return NMS_ERR_WORKSPACE;
    g_pool.ws = workspace;
    g_pool.bytes = ws_bytes;
    g_pool.n_max = n_max;
    g_pool.frames_max = frames_max;
    return NMS_OK;
}

int nms_shutdown(void)
{
    g_pool = Pool();
    return NMS_OK;
}

int nms_run(const float *boxes, const float *scores, int n, float threshold, uint8_t *keep_out, void *stream)
{
    int st;
    if (!sizes_ok(n, 1, &st)) return st;
    if (is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    if (n == 0) return NMS_OK;
    if (!g_pool.ws || n > g_pool.n_max) return NMS_ERR_WORKSPACE;
    return nms_run_batched(boxes, scores, nullptr, n, 1, threshold, keep_out, g_pool.ws, g_pool.bytes, stream);
}

int nms_host_pair_test(const float *victim, const float *outranking, float threshold)
{
    if (!victim || !outranking || is_nan(threshold)) return NMS_ERR_INVALID_ARG;
    const NmsThetaConst th = nms_make_theta_const(threshold);
    const float a = nms_box_area(outranking[0], outranking[1], outranking[2], outranking[3]);
    bool hit;
    const bool regular = nms_y_regular(victim[1]) && nms_y_regular(victim[3]) && nms_y_regular(outranking[1]) &&
                         nms_y_regular(outranking[3]);
    if (th.fast && regular)  // what the fused kernel does for a pair of regular tiles
        hit = nms_eliminates_fast_yscaled(victim[0], victim[1] * NMS_YSCALE, victim[2], victim[3] * NMS_YSCALE,
                                          outranking[0], outranking[1] * NMS_YSCALE, outranking[2],
                                          outranking[3] * NMS_YSCALE, nms_pair_threshold(a, th.m) * NMS_YSCALE, NMS_YSCALE);
    else if (th.fast)
        hit = nms_eliminates_fast(victim[0], victim[1], victim[2], victim[3],
                                  outranking[0], outranking[1], outranking[2], outranking[3], nms_pair_threshold(a, th.m));
    else
        hit = nms_eliminates_exact(victim[0], victim[1], victim[2], victim[3],
                                   outranking[0], outranking[1], outranking[2], outranking[3], a, th.theta);
    return hit ? 1 : 0;
}

}  // extern "C"
