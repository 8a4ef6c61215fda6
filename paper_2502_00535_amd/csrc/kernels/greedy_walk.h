// Part of nms_kernels.hip (included there, inside its anonymous namespace): classic greedy rule without a mask: one workgroup walks a frame in rank order (also with the variants).
#pragma once

// ----------------------------------------------------------------------------- greedy rule without a mask

// The classic sequential rule walked tile by tile in rank order, one workgroup (16
// wavefronts) per frame, no mask in memory.  Under this rule a box that is eliminated
// neither eliminates others nor needs any further test, so only the SURVIVORS are ever used
// as outranking boxes: about 600 of 4096 on frames like configuration 4, i.e. a seventh of
// the pair grid.  A frame is one compute unit's work, so the route pays from a few dozen
// frames on.
//
// The rows that are left (at first all of them) are numbered in rank order and cut into tiles
// of 64; wavefront w owns the tiles w, w + 16, w + 32, w + 48 and keeps their boxes in
// registers, lane = row, with one wave-uniform 64-bit word per tile for the rows that are out.
// Round t settles tile t, whose rows its owner has put into LDS:
//   - all wavefronts, a share each: the survivors of tile t-1 ("list t-1", in LDS) against the
//     tile, and for each row of the tile the better-ranked rows of the tile itself that
//     eliminate it (one 64-bit word per row); barrier;
//   - the owner combines the shares and finds the tile's survivors as the fixed point of
//     "alive, and not eliminated by a surviving better-ranked row of the tile", writes them
//     to LDS as list t and marks them in keep_out; meanwhile every wavefront applies list t-1
//     to all its other tiles; barrier.
//
// Most rows that die do so early (on configuration 4 more than half of the rows are out after
// the first two tiles), and a tile costs the same with one row alive as with 64.  So the walk
// runs in stages of 2, 4, 8, ... tiles; after a stage the rows still alive are compacted (their
// rank numbers through LDS, their boxes gathered again from the table) into fewer tiles and
// the walk starts over on them.  The last stage begins once 16 tiles or fewer are left.
constexpr int kFusedWaves = 16;
constexpr int kFusedOwned = NMS_SORT_CHUNK / kTile / kFusedWaves;  // 4
constexpr long long kGreedyFusedBoxes = 32ll * 4096;  // nms_run_greedy_batched takes this route from frames * n_max boxes on

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

// Bitwise OR over each row of 16 lanes, in the row's last lane.
__device__ __forceinline__ unsigned row_or16(unsigned x)
{
    x |= (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x111, 0xf, 0xf, true);  // row_shr:1
    x |= (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x112, 0xf, 0xf, true);  // row_shr:2
    x |= (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x114, 0xf, 0xf, true);  // row_shr:4
    x |= (unsigned)__builtin_amdgcn_update_dpp(0, (int)x, 0x118, 0xf, 0xf, true);  // row_shr:8
    return x;
}

constexpr int kWalkChunk = 4;  // survivors fetched from LDS at a time
constexpr int kWalkLists = 2;  // lists kept in LDS: the one being written and the one being applied

template <bool EX, bool IOU, int MODE, bool AUX>
__global__ void __launch_bounds__(kFusedWaves * 64)
greedy_fused_kernel(const float *__restrict__ sorted5, const int32_t *__restrict__ order,
                    const int32_t *__restrict__ counts, int n_max, int n_pad, NmsThetaConst th, FusedVariant opt,
                    uint8_t *__restrict__ keep_out)
{
    constexpr bool kUseT = MODE == kExBoundary && !IOU;  // the list carries T, else the area
    constexpr int kTileBuf = kWalkLists;                 // one more buffer of the same layout: the rows of the tile being settled
    __shared__ float4 box_s[kWalkLists + 1][kTile];      // list t in buffer t % kWalkLists
    __shared__ float aux_s[kWalkLists + 1][kTile];
    __shared__ float score_s[kWalkLists + 1][kTile];
    __shared__ int label_s[kWalkLists + 1][kTile];
    __shared__ int count_s[kWalkLists];
    __shared__ unsigned long long part_s[kFusedWaves];   // rows of the tile being settled that a wavefront's share of the list before eliminates
    __shared__ unsigned long long hitters_s[kTile];      // per row of that tile: the better-ranked rows of the tile that eliminate it
    __shared__ int alive_s[NMS_SORT_CHUNK / kTile];  // compaction: rows alive per tile
    __shared__ int ids_s[NMS_SORT_CHUNK];            // compaction: rank numbers of the rows left
    const int f = blockIdx.x;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int n_f = frame_count(counts, f, n_max);
    const float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    const float4 *box4 = reinterpret_cast<const float4 *>(sorted_f);
    const float *area = sorted_f + 4 * (size_t)n_pad;
    uint8_t *keep_f = keep_out + (size_t)f * n_max;
    const int32_t *order_f = order + (size_t)f * n_max;

    for (int i = (int)threadIdx.x; i < n_max; i += blockDim.x) keep_f[i] = 0;  // survivors are marked as they are found

    // The owned tiles that are not settled yet, the next one to settle in slot 0 (after a tile is
    // settled the others move down one slot).
    float4 vb[kFusedOwned];
    FusedCandidate self[kFusedOwned];     // the same rows in their role as outranking boxes
    int rank_of[kFusedOwned];             // rank number of the lane's row
    unsigned long long out[kFusedOwned];  // wave-uniform; bit r: row r is eliminated or does not exist
    int left = 0;                         // owned tiles not settled yet
    int tn = 0;                           // number of the tile in slot 0 (the others follow in steps of 16)
    int n_cur = n_f;                      // rows in the current numbering

    // (re)load the owned tiles of the current numbering; `compacted`: rank numbers come from ids_s
    auto load_tiles = [&](bool compacted) __attribute__((always_inline)) {
        left = 0;
        tn = wave;
#pragma unroll
        for (int i = 0; i < kFusedOwned; ++i) {
            const int first = (wave + kFusedWaves * i) * kTile;
            const bool has = first < n_cur;
            left += has ? 1 : 0;
            const int q = first + lane;
            const bool real = q < n_cur;
            const int r = real ? (compacted ? ids_s[q] : q) : 0;  // rows that do not exist read row 0 and are marked out
            rank_of[i] = r;
            vb[i] = box4[r];
            FusedCandidate me;
            me.x1 = vb[i].x, me.y1 = vb[i].y, me.x2 = vb[i].z, me.y2 = vb[i].w;
            me.area = EX ? ((vb[i].z - vb[i].x) + opt.offset) * ((vb[i].w - vb[i].y) + opt.offset) : area[r];
            me.T = MODE == kExBoundary ? nms_pair_threshold(me.area, EX ? opt.boundary : th.m) : 0.0f;
            me.score = AUX ? opt.ranked_score[(size_t)f * n_pad + r] : 0.0f;
            me.label = (AUX && (opt.flags & kExClasses)) ? opt.ranked_label[(size_t)f * n_pad + r] : 0;
            self[i] = me;
            out[i] = !has ? ~0ull : (first + kTile <= n_cur ? 0ull : ~0ull << (n_cur - first));
        }
    };
    load_tiles(false);
    __syncthreads();  // the zero fill is complete before any survivor's byte is written

    // Entry k of buffer `buf` (a list's survivor, or a row of the tile being settled).  With a
    // wave-uniform k every lane gets the same entry (a broadcast read); with k = lane, its own.
    auto entry = [&](int buf, int k) __attribute__((always_inline)) {
        FusedCandidate c;
        const float4 b = box_s[buf][k];
        c.x1 = b.x, c.y1 = b.y, c.x2 = b.z, c.y2 = b.w;
        c.T = kUseT ? aux_s[buf][k] : 0.0f;
        c.area = kUseT ? 0.0f : aux_s[buf][k];
        c.score = AUX ? score_s[buf][k] : 0.0f;
        c.label = AUX ? label_s[buf][k] : 0;
        return c;
    };
    // The list in buffer `buf` against the tiles in slots 0 .. N-1.  Survivors are fetched four
    // at a time into two sets of registers in turn, the next four while the current four are
    // tested; a full chunk has no branch inside.
    auto apply_slots = [&](auto slots, int buf) __attribute__((always_inline)) {
        constexpr int N = decltype(slots)::value;
        const int count = __builtin_amdgcn_readfirstlane(count_s[buf]);
        if (count == 0) return;
        auto fetch = [&](FusedCandidate (&c)[kWalkChunk], int k0) __attribute__((always_inline)) {
#pragma unroll
            for (int u = 0; u < kWalkChunk; ++u) c[u] = entry(buf, k0 + u < count ? k0 + u : count - 1);
        };
        auto test = [&](const FusedCandidate (&c)[kWalkChunk], int k0) __attribute__((always_inline)) {
            if (k0 + kWalkChunk <= count) {
#pragma unroll
                for (int u = 0; u < kWalkChunk; ++u) {
#pragma unroll
                    for (int i = 0; i < N; ++i)
                        out[i] |= __ballot(fused_hit<EX, IOU, MODE, AUX>(vb[i], self[i].area, self[i].score, self[i].label,
                                                                          c[u], th.theta, opt));
                }
            } else {
#pragma unroll
                for (int u = 0; u < kWalkChunk - 1; ++u) {
                    if (k0 + u < count) {  // wave-uniform
#pragma unroll
                        for (int i = 0; i < N; ++i)
                            out[i] |= __ballot(fused_hit<EX, IOU, MODE, AUX>(vb[i], self[i].area, self[i].score,
                                                                              self[i].label, c[u], th.theta, opt));
                    }
                }
            }
        };
        FusedCandidate even[kWalkChunk], odd[kWalkChunk];
        fetch(even, 0);
        for (int k0 = 0; k0 < count; k0 += 2 * kWalkChunk) {
            if (k0 + kWalkChunk < count) fetch(odd, k0 + kWalkChunk);
            test(even, k0);
            if (k0 + kWalkChunk >= count) break;
            if (k0 + 2 * kWalkChunk < count) fetch(even, k0 + 2 * kWalkChunk);
            test(odd, k0 + kWalkChunk);
        }
    };
    auto apply = [&](int slots, int buf) __attribute__((always_inline)) {  // the same for a number of slots known at run time
        if (slots == 1) apply_slots(std::integral_constant<int, 1>(), buf);
        else if (slots == 2) apply_slots(std::integral_constant<int, 2>(), buf);
        else if (slots == 3) apply_slots(std::integral_constant<int, 3>(), buf);
        else if (slots >= 4) apply_slots(std::integral_constant<int, 4>(), buf);
    };
    static_assert(kFusedOwned == 4, "apply() dispatches on up to four slots");

    // the rows of slot 0 into LDS for the round that settles them
    auto post_tile = [&]() __attribute__((always_inline)) {
        box_s[kTileBuf][lane] = vb[0];
        aux_s[kTileBuf][lane] = kUseT ? self[0].T : self[0].area;
        if (AUX) score_s[kTileBuf][lane] = self[0].score;
        if (AUX) label_s[kTileBuf][lane] = self[0].label;
    };

    int g = 0;          // rounds so far over all stages: round g writes list g, into buffer g % kWalkLists
    for (int stage_tiles = 2;; stage_tiles *= 2) {
        const int tiles_cur = (n_cur + kTile - 1) / kTile;
        const int rounds = (tiles_cur <= kFusedWaves || stage_tiles >= tiles_cur) ? tiles_cur : stage_tiles;
        if (wave == 0) post_tile();  // tile 0 of this numbering
        lds_barrier();
        for (int t = 0; t < rounds; ++t, ++g) {
            const int pending = (g - 1) & (kWalkLists - 1);  // buffer of the list before (there is none in the very first round)
            // All wavefronts, a share each, on the tile being settled (its rows are in LDS, lane =
            // row): the survivors of the list before against it, and for each of its rows the
            // better-ranked rows of the tile itself that eliminate it.
            {
                const FusedCandidate row = entry(kTileBuf, lane);
                const float4 row_box = make_float4(row.x1, row.y1, row.x2, row.y2);
                const int count = g > 0 ? __builtin_amdgcn_readfirstlane(count_s[pending]) : 0;
                unsigned long long part = 0;
                for (int k = wave; k < count; k += kFusedWaves)
                    part |= __ballot(fused_hit<EX, IOU, MODE, AUX>(row_box, row.area, row.score, row.label, entry(pending, k),
                                                                    th.theta, opt));
                if (lane == 0) part_s[wave] = part;
                FusedCandidate victim[kTile / kFusedWaves];
#pragma unroll
                for (int j = 0; j < kTile / kFusedWaves; ++j) victim[j] = entry(kTileBuf, wave + kFusedWaves * j);
#pragma unroll
                for (int j = 0; j < kTile / kFusedWaves; ++j) {
                    const int r = wave + kFusedWaves * j;
                    const bool hit = fused_hit<EX, IOU, MODE, AUX>(make_float4(victim[j].x1, victim[j].y1, victim[j].x2, victim[j].y2),
                                                                   victim[j].area, victim[j].score, victim[j].label, row,
                                                                   th.theta, opt) &&
                                     lane < r;
                    const unsigned long long hitters = __ballot(hit);
                    if (lane == 0) hitters_s[r] = hitters;
                }
            }
            lds_barrier();
            if (wave == (t & (kFusedWaves - 1))) {
                // Settle tile t (slot 0).  A row survives iff it is alive and no surviving
                // better-ranked row of the tile eliminates it; iterated from "every alive row
                // survives" this settles one more row per pass at least, in practice a few passes.
                __builtin_amdgcn_s_setprio(3);
                const unsigned long long share = part_s[lane & (kFusedWaves - 1)];
                const unsigned dead_lo = row_or16((unsigned)share), dead_hi = row_or16((unsigned)(share >> 32));
                const unsigned long long dead =
                    out[0] | ((unsigned long long)(unsigned)__builtin_amdgcn_readlane((int)dead_hi, kFusedWaves - 1) << 32) |
                    (unsigned)__builtin_amdgcn_readlane((int)dead_lo, kFusedWaves - 1);
                const unsigned long long hitters = hitters_s[lane];
                const bool alive = ((~dead >> lane) & 1ull) != 0;
                unsigned long long kept = ~dead;
                for (int pass = 0; pass < kTile; ++pass) {
                    const unsigned long long next = __ballot(alive && (hitters & kept) == 0);
                    if (next == kept) break;
                    kept = next;
                }
                const float4 v = vb[0];
                const FusedCandidate mine = self[0];
                const bool is_kept = (kept >> lane) & 1ull;
                const int into = g & (kWalkLists - 1);
                if (is_kept) {  // survivor number k of the tile is entry k of the list
                    const int k = __builtin_popcountll(kept & ((1ull << lane) - 1ull));
                    box_s[into][k] = v;
                    aux_s[into][k] = kUseT ? mine.T : mine.area;
                    if (AUX) score_s[into][k] = mine.score;
                    if (AUX) label_s[into][k] = mine.label;
                }
                if (lane == 0) count_s[into] = __builtin_popcountll(kept);
                __builtin_amdgcn_s_setprio(0);
                if (is_kept) keep_f[order_f[rank_of[0]]] = 1;
#pragma unroll
                for (int i = 0; i + 1 < kFusedOwned; ++i) {
                    vb[i] = vb[i + 1];
                    self[i] = self[i + 1];
                    rank_of[i] = rank_of[i + 1];
                    out[i] = out[i + 1];
                }
                --left;
                tn += kFusedWaves;
            } else if (t + 1 < rounds && wave == ((t + 1) & (kFusedWaves - 1))) {
                post_tile();  // the next round's tile
            }
            if (g > 0) apply(left, pending);  // the list before against the tiles that are left
            lds_barrier();
        }
        if (rounds == tiles_cur) break;  // every tile is settled

        // End of a stage: the rows still alive move together (the list just written has not been
        // applied yet; it holds boxes, not row numbers, and is applied in the next stage's first
        // round like any other).  Tile `rounds + j` of the old numbering reports its count in
        // alive_s[j]; a prefix sum gives every tile its place in ids_s.
        const int tiles_left = tiles_cur - rounds;
#pragma unroll
        for (int i = 0; i < kFusedOwned; ++i) {
            if (i < left && lane == 0) alive_s[tn - rounds + kFusedWaves * i] = __builtin_popcountll(~out[i]);
        }
        lds_barrier();
        const unsigned mine_alive = lane < tiles_left ? (unsigned)alive_s[lane] : 0u;
        const unsigned incl = wave_inclusive_sum(mine_alive);
        const int total = __builtin_amdgcn_readlane((int)incl, 63);
#pragma unroll
        for (int i = 0; i < kFusedOwned; ++i) {
            if (i < left) {  // wave-uniform
                const int base = __builtin_amdgcn_readlane((int)(incl - mine_alive), tn - rounds + kFusedWaves * i);
                const unsigned long long alive = ~out[i];
                if ((alive >> lane) & 1ull) ids_s[base + __builtin_popcountll(alive & ((1ull << lane) - 1ull))] = rank_of[i];
            }
        }
        lds_barrier();
        n_cur = total;
        load_tiles(true);
    }
}
