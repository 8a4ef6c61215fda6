// Part of nms_kernels.hip (included there, inside its anonymous namespace): frames of at most 1024 boxes, rank step and two stages of pair tests in one launch.
#pragma once

// ----------------------------------------------------------------------------- small frames, one launch

// A batch of some tens to hundreds of frames of at most a thousand boxes is too much arithmetic
// for the direct form and too little for separate launches: the rank kernel keeps one compute
// unit per frame busy for 8 us and hands its tables over through memory to a map launch that
// needs 2 us to get going.  Here one workgroup does everything for its frame and the ranked table
// never leaves LDS; and since V_i is the AND over all j (section "Algorithm Correctness"), a victim
// that has met one eliminator needs no further test, which on clustered detections is most victims
// after the best-ranked boxes have been tried:
//
//   rank      Algorithm 1's order "D[i].s < D[j].s" (ties by index): thread e holds box and key of
//             input element e, the workgroup sorts the keys (radix_rank_one, slots beyond the frame's
//             count last), the boxes change hands through LDS and thread r builds row r of the table (box, y scaled
//             when every box of the frame allows it; its decision threshold T, or its area for
//             thresholds that take the literal division; its input index);
//   stage 1   every victim of the workgroup against the best kSmallFirst ranks: lane = victim, two
//             victims per lane (two tiles of 64), the outranking boxes read from the table as
//             broadcasts, eight per work item -- a broadcast moves 64 x 16 bytes whatever it is
//             used for, and with one victim per lane the LDS path, not the VALU, would set the
//             pace; the compare's lane mask is the set of victims the box eliminates, ORed up in
//             a scalar register and merged per victim tile in LDS;
//   pack      victims with an eliminator, and victims ranked inside the first stage's boxes, are
//             final and written out; the others are listed in rank order;
//   stage 2   the listed victims against the remaining tiles: lane = outranking box, four tiles
//             per wavefront in registers, the victims read as broadcasts (one read per four rows);
//             a tile counts from the rank of its first box on, the tile that holds the victim's
//             own rank up to that rank.
//
// With fewer frames than compute units a frame is given to `parts` workgroups: each sorts the
// whole frame (the sort is bound by latency, not by work: the copies cost nothing while the other
// compute units would idle) and takes the victims of ranks part, part + parts, ... -- interleaved
// ranks give every share the same mix of early and late victims.  Each victim's keep byte is
// written once, by its workgroup.  Same keep vector as the all-pairs routes, bit for bit: a victim
// is dropped only once an eliminator has been found.
constexpr int kSmallWaves = 16;
constexpr int kSmallThreads = kSmallWaves * 64;
constexpr int kSmallFirst = 128;  // outranking boxes of the first stage
constexpr int kSmallGroup = 8;    // outranking boxes per work item of the first stage
constexpr int kSmallTiles = 4;    // tiles a wavefront holds in registers in the second stage

template <int PAIR>
__device__ __forceinline__ bool small_hit(const float4 v, const float4 c, float aux, float theta, float y_one)
{
    if (PAIR == kPairFastYScaled) return nms_eliminates_fast_yscaled(v.x, v.y, v.z, v.w, c.x, c.y, c.z, c.w, aux, y_one);
    if (PAIR == kPairFast) return nms_eliminates_fast(v.x, v.y, v.z, v.w, c.x, c.y, c.z, c.w, aux);
    return nms_eliminates_exact(v.x, v.y, v.z, v.w, c.x, c.y, c.z, c.w, aux, theta);
}

// Stage 1, one work item: the outranking ranks [c0, c0 + kSmallGroup) against R victim tiles (this
// lane's victims v[] of ranks r[]).  GUARD: the first so many tiles of the set hold victims ranked at
// or before some of the boxes, so there a box counts only for the lanes whose victim is ranked behind it.
template <int PAIR, int GUARD, int R>
__device__ __forceinline__ void small_first_item(const float4 *tbox, const float *taux, int c0, const float4 (&v)[R],
                                                 const int (&r)[R], float theta, float y_one, unsigned long long (&dead)[R])
{
    // four boxes at a time: with all eight in flight next to four victims' chains the kernel runs out of registers
#pragma unroll
    for (int half = 0; half < kSmallGroup; half += 4) {
        float4 cb[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) cb[k] = tbox[c0 + half + k];
        const float4 a4 = *reinterpret_cast<const float4 *>(taux + c0 + half);
        const float ca[4] = {a4.x, a4.y, a4.z, a4.w};
#pragma unroll
        for (int k = 0; k < 4; ++k) {
#pragma unroll
            for (int q = 0; q < R; ++q) {
                unsigned long long h = __ballot(small_hit<PAIR>(v[q], cb[k], ca[k], theta, y_one));
                if (q < GUARD) h &= __ballot(r[q] > c0 + half + k);
                dead[q] |= h;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Stage 1 for the workgroup's victim tiles in sets of R: items (set, group of kSmallGroup boxes) dealt
// round-robin to the wavefronts; a set's eliminated victims are merged per tile in dead1[].
template <int PAIR, int R>
__device__ __forceinline__ void small_first_stage(const float4 *tbox, const float *taux, unsigned long long *dead1, int m0,
                                                  int first, int part, int parts, float theta, float y_one)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int vtiles = (m0 + kTile - 1) / kTile;
    const int sets = (vtiles + R - 1) / R;
    const int groups = first / kSmallGroup;
    for (int item = wave; item < sets * groups; item += kSmallWaves) {
        const int set = item / groups;
        const int c0 = (item % groups) * kSmallGroup;
        float4 v[R];
        int r[R];
        unsigned long long dead[R];
#pragma unroll
        for (int q = 0; q < R; ++q) {
            const int i = (R * set + q) * kTile + lane;
            r[q] = i < m0 ? part + parts * i : 0;  // a lane beyond the share tests row 0: its bits are never read
            v[q] = tbox[r[q]];
            dead[q] = 0ull;
        }
        // a tile's lowest rank is that of its first lane; the ranks rise from tile to tile
        int guarded = 0;
        while (guarded < R && part + parts * (R * set + guarded) * kTile < c0 + kSmallGroup) ++guarded;
        if (guarded == 0)
            small_first_item<PAIR, 0, R>(tbox, taux, c0, v, r, theta, y_one, dead);
        else if (guarded == 1)
            small_first_item<PAIR, 1, R>(tbox, taux, c0, v, r, theta, y_one, dead);
        else
            small_first_item<PAIR, 2, R>(tbox, taux, c0, v, r, theta, y_one, dead);  // ranks < 128: at most the first two tiles
        if (lane == 0) {
#pragma unroll
            for (int q = 0; q < R; ++q)
                if (dead[q] != 0ull && R * set + q < vtiles) atomicOr(&dead1[R * set + q], dead[q]);
        }
    }
}

// Stage 2, one victim (rank r, box v, read as broadcasts) against the tiles t0 .. t0 + 3 held in
// cb[], aux[]: is there an eliminator among the boxes ranked before r?  Branch-free, so that the
// tests of several victims can be interleaved.  MASKED: the victim's rank lies inside the group's
// tiles (or the group has fewer than four), so every tile's lane mask is cut down to the boxes ranked
// before r (all, the lower r - 64 t lanes of the tile that holds rank r, none; a tile beyond the
// frame's last is a copy of tile t0 with an empty mask).  Otherwise all four tiles are ranked before
// r: the scalar unit, which the four SIMDs share, then has one instruction per row to do, not twelve.
template <int PAIR, bool MASKED>
__device__ __forceinline__ bool small_second_victim(const float4 v, int r, const float4 (&cb)[kSmallTiles],
                                                    const float (&aux)[kSmallTiles], int t0, int useful, float theta, float y_one)
{
    unsigned long long any = 0ull;
#pragma unroll
    for (int j = 0; j < kSmallTiles; ++j) {
        unsigned long long h = __ballot(small_hit<PAIR>(v, cb[j], aux[j], theta, y_one));
        if (MASKED) {
            int before = r - (t0 + j) * kTile;  // boxes of tile t0 + j ranked before the victim
            before = before < 0 ? 0 : (before > kTile ? kTile : before);
            if (j >= useful) before = 0;
            h &= before >= kTile ? ~0ull : (1ull << before) - 1ull;
        }
        any |= h;
    }
    return any != 0ull;
}

// A unit of stage 2: the listed victims [k_begin, k_end) against the tiles in cb[], aux[], four at a
// time, their reads issued together (a short last batch repeats its last victim).  (Requesting the
// next four while these are tested measured slower.)
template <int PAIR, bool MASKED>
__device__ __forceinline__ void small_second_unit(const float4 *tbox, const int *list, unsigned char *flag2, int k_begin, int k_end,
                                                  const float4 (&cb)[kSmallTiles], const float (&aux)[kSmallTiles], int t0,
                                                  int useful, float theta, float y_one)
{
    const int lane = threadIdx.x & 63;
#pragma unroll 1
    for (int k = k_begin; k < k_end; k += 4) {
        int at[4], r[4];
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            at[u] = k + u < k_end ? k + u : k_end - 1;
            r[u] = list[at[u]];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            r[u] = __builtin_amdgcn_readfirstlane(r[u]);
            v[u] = tbox[r[u]];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const bool dead = small_second_victim<PAIR, MASKED>(v[u], r[u], cb, aux, t0, useful, theta, y_one);
            if (lane == 0 && dead) flag2[at[u]] = 1;
        }
    }
}

// The stages of one workgroup.  The table (tbox, taux) holds the frame in rank order; the workgroup's
// victims are the ranks part + parts * i, i < m0.  Writes keep_f through tord (rank -> input index).
template <int PAIR>
__device__ __forceinline__ void small_stages(const float4 *tbox, const float *taux, const int *tord, unsigned long long *dead1,
                                             int *list, unsigned char *flag2, int *wcount, int n_f, int part, int parts,
                                             float theta, float y_one, uint8_t *keep_f)
{
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tiles_f = (n_f + kTile - 1) / kTile;
    const int m0 = n_f > part ? (n_f - part + parts - 1) / parts : 0;
    const int first = tiles_f * kTile < kSmallFirst ? tiles_f * kTile : kSmallFirst;  // boxes of stage 1 (padding rows included)

    // ---- stage 1: four victims per lane where the share has three tiles or more (a broadcast of an outranking
    // box then serves four rows), two otherwise (fewer idle lanes)
    if ((m0 + kTile - 1) / kTile > 2)
        small_first_stage<PAIR, 4>(tbox, taux, dead1, m0, first, part, parts, theta, y_one);
    else
        small_first_stage<PAIR, 2>(tbox, taux, dead1, m0, first, part, parts, theta, y_one);
    __syncthreads();

    // ---- pack: final victims are written out, the others listed in rank order
    int r_mine = 0;
    bool alive = false;
    if (tid < m0) {
        r_mine = part + parts * tid;
        const bool dead = ((dead1[tid / kTile] >> (tid % kTile)) & 1ull) != 0ull;
        if (dead || r_mine <= first)
            keep_f[tord[r_mine]] = dead ? 0 : 1;  // every box ranked before r_mine was among the first stage's
        else
            alive = true;
    }
    // (counted here as well: per tile group of stage 2, the listed victims ranked at or before the group's
    // first box -- they have nothing to meet in it, and the list being in rank order they come first)
    const unsigned long long alive_mask = __ballot(alive);
    const int t_begin = first / kTile;
    if (lane == 0) wcount[wave] = (int)__popcll(alive_mask);
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        const int n = (int)__popcll(__ballot(alive && r_mine <= (t_begin + g * kSmallTiles) * kTile));
        if (lane == 0) wcount[kSmallWaves * (g + 1) + wave] = n;
    }
    __syncthreads();
    // the five rows of sixteen counts summed by every wavefront for itself: a lane per count, prefix sums inside
    // the rows of sixteen lanes (DPP), totals read from each row's last lane
    const int sums_a = (int)row16_inclusive_sum((unsigned)wcount[lane]);
    const int sums_b = (int)row16_inclusive_sum((unsigned)wcount[kTile + (lane & 15)]);
    const int listed = __builtin_amdgcn_readlane(sums_a, 15);
    const int before = wave == 0 ? 0 : __builtin_amdgcn_readlane(sums_a, wave - 1);
    int start[4] = {__builtin_amdgcn_readlane(sums_a, 31), __builtin_amdgcn_readlane(sums_a, 47), __builtin_amdgcn_readlane(sums_a, 63),
                    __builtin_amdgcn_readlane(sums_b, 15)};
    if (alive) {
        const int pos = before + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(alive_mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)alive_mask, 0u));
        list[pos] = r_mine;
        flag2[pos] = 0;
    }
    __syncthreads();

    // ---- stage 2: tiles first / 64 .. tiles_f - 1 in groups of kSmallTiles.  The list is in rank order, so a
    // group meets only the victims from list position start[g] on.
    const int groups2 = (tiles_f - t_begin + kSmallTiles - 1) / kSmallTiles;  // at most 4: P / 64 - 2 tiles
    if (listed > 0 && listed <= kTile && groups2 > 0) {
        // A short list (clustered detections): a unit is (group, four consecutive listed victims), the units of
        // all groups in one numbering dealt round-robin to the wavefronts.
        int units_before[5];
        units_before[0] = 0;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            if (g >= groups2) start[g] = listed;
            units_before[g + 1] = units_before[g] + (listed - start[g] + 3) / 4;
        }
        for (int unit = wave; unit < units_before[4]; unit += kSmallWaves) {
            int g = 0;
#pragma unroll
            for (int q = 1; q < 4; ++q) g += unit >= units_before[q] ? 1 : 0;
            const int k_begin = (g == 0 ? start[0] : g == 1 ? start[1] : g == 2 ? start[2] : start[3]) +
                                4 * (unit - (g == 0 ? units_before[0] : g == 1 ? units_before[1] : g == 2 ? units_before[2] : units_before[3]));
            const int t0 = t_begin + g * kSmallTiles;
            const int useful = tiles_f - t0 < kSmallTiles ? tiles_f - t0 : kSmallTiles;
            // four victims, their reads issued together (a short last unit repeats its last victim)
            int at[4], r[4];
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                at[u] = k_begin + u < listed ? k_begin + u : listed - 1;
                r[u] = list[at[u]];
            }
            float4 cb[kSmallTiles];
            float aux[kSmallTiles];
#pragma unroll
            for (int j = 0; j < kSmallTiles; ++j) {
                const int row = (t0 + (j < useful ? j : 0)) * kTile + lane;
                cb[j] = tbox[row];
                aux[j] = taux[row];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                r[u] = __builtin_amdgcn_readfirstlane(r[u]);
                v[u] = tbox[r[u]];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const bool dead = small_second_victim<PAIR, true>(v[u], r[u], cb, aux, t0, useful, theta, y_one);
                if (lane == 0 && dead) flag2[at[u]] = 1;
            }
        }
    }
    if (listed > kTile && groups2 > 0) {
        // A long list (little was eliminated).  From list position start[g + 1] on the victims are ranked behind all
        // tiles of group g: two ranges per group (ranks inside the group's tiles: lane masks needed; beyond: none),
        // each cut into units of `span` consecutive victims -- about two units per wavefront, so that a group's
        // tiles are fetched once for many victims.
        int range_begin[8], range_end[8], units_before[9];
        int slots = 0;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int from = g < groups2 ? start[g] : listed;
            const int full_group = (t_begin + (g + 1) * kSmallTiles) <= tiles_f;  // a group cut short by the frame's end keeps its masks
            const int beyond = g + 1 < groups2 && full_group ? start[g + 1] : listed;
            range_begin[2 * g] = from;
            range_end[2 * g] = beyond;
            range_begin[2 * g + 1] = beyond;
            range_end[2 * g + 1] = listed;
            slots += listed - from;
        }
        int span = (slots + 2 * kSmallWaves - 1) / (2 * kSmallWaves);
        span = span < 4 ? 4 : (span + 3) / 4 * 4;
        units_before[0] = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) units_before[i + 1] = units_before[i] + (range_end[i] - range_begin[i] + span - 1) / span;
        for (int unit = wave; unit < units_before[8]; unit += kSmallWaves) {
            int i = 0;
#pragma unroll
            for (int q = 1; q < 8; ++q) i += unit >= units_before[q] ? 1 : 0;
            int first_unit = 0, from = 0, to = 0;
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                if (q == i) {
                    first_unit = units_before[q];
                    from = range_begin[q];
                    to = range_end[q];
                }
            }
            const int k_begin = from + span * (unit - first_unit);
            const int k_end = k_begin + span < to ? k_begin + span : to;
            const int t0 = t_begin + (i / 2) * kSmallTiles;
            const int useful = tiles_f - t0 < kSmallTiles ? tiles_f - t0 : kSmallTiles;
            float4 cb[kSmallTiles];
            float aux[kSmallTiles];
#pragma unroll
            for (int j = 0; j < kSmallTiles; ++j) {
                const int row = (t0 + (j < useful ? j : 0)) * kTile + lane;
                cb[j] = tbox[row];
                aux[j] = taux[row];
            }
            if ((i & 1) == 0)
                small_second_unit<PAIR, true>(tbox, list, flag2, k_begin, k_end, cb, aux, t0, useful, theta, y_one);
            else
                small_second_unit<PAIR, false>(tbox, list, flag2, k_begin, k_end, cb, aux, t0, useful, theta, y_one);
        }
    }
    __syncthreads();
    for (int k = tid; k < listed; k += kSmallThreads) keep_f[tord[list[k]]] = flag2[k] ? 0 : 1;
}

// n_max <= kSmallThreads.  FAST: the threshold has a division-free form (NmsThetaConst).
// Grid: frames * parts workgroups of kSmallThreads threads.
template <bool FAST>
__global__ void __launch_bounds__(kSmallThreads)
small_frames_kernel(const float *__restrict__ boxes, const float *__restrict__ scores, const int32_t *__restrict__ counts,
                    int n_max, int parts, NmsThetaConst th, uint8_t *__restrict__ keep_out)
{
    constexpr int P = kSmallThreads;  // rows of the table: one per thread
    __shared__ unsigned long long keys[P];
    __shared__ __align__(16) unsigned hist[kSmallWaves * 256];
    __shared__ __align__(16) unsigned wbase[kSmallWaves * 256];
    __shared__ __align__(16) unsigned tot[256];
    __shared__ float4 stage[2 * P];  // the sort's lane-mask tables, then the boxes in input order
    __shared__ float saux[P];        // and their decision values
    __shared__ float4 tbox[P];
    __shared__ __align__(16) float taux[P];
    __shared__ int tord[P];
    __shared__ unsigned long long dead1[P / kTile];
    __shared__ int list[P];
    __shared__ unsigned char flag2[P];
    __shared__ int wcount[5 * kSmallWaves];  // per wavefront: listed victims, and those before each of stage 2's tile groups
    const int f = blockIdx.x / parts;
    const int part = blockIdx.x % parts;
    const int tid = (int)threadIdx.x;
    const int n_f = frame_count(counts, f, n_max);
    const float *scores_f = scores + (size_t)f * n_max;
    const float4 *boxes_f = reinterpret_cast<const float4 *>(boxes + (size_t)f * n_max * 4);
    uint8_t *keep_f = keep_out + (size_t)f * n_max;

    // rank: thread e holds element e of the input (slots beyond the frame's count sort to the end)
    float4 mine = make_float4(0.f, 0.f, 0.f, 0.f);
    unsigned long long key = kSentinel;
    if (tid < n_f) {
        mine = boxes_f[tid];
        key = nms_rank_key(scores_f[tid], (unsigned)tid);
    }
    // what the table needs per box is worked out here, in input order, while the loads are the only thing in flight:
    // does every y of the frame allow the scaled form (slots beyond the count hold the box (0,0,0,0), which does), and
    // the box's decision value (no intersection reaches a padding row's)
    const bool odd = !(nms_y_regular(mine.y) && nms_y_regular(mine.w));
    const bool scaled = FAST && __syncthreads_or(odd ? 1 : 0) == 0;
    const float area = nms_box_area(mine.x, mine.y, mine.z, mine.w);
    float mine_aux = FAST ? (tid < n_f ? nms_pair_threshold(area, th.m) : INFINITY) : area;
    if (scaled) {
        mine.y *= NMS_YSCALE;
        mine.w *= NMS_YSCALE;
        mine_aux *= NMS_YSCALE;
    }
    radix_rank_one<kSmallWaves>((unsigned)(key >> 32), (unsigned)key, keys, hist, tot, wbase, reinterpret_cast<unsigned long long *>(stage));
    stage[tid] = mine;
    saux[tid] = mine_aux;
    if (tid < P / kTile) dead1[tid] = 0ull;
    __syncthreads();
    {
        // row tid of the table: the box of rank tid, or the padding row (the input's slot tid: it holds one too)
        const int idx = tid < n_f ? (int)(unsigned)keys[tid] : tid;
        tbox[tid] = stage[idx];
        taux[tid] = saux[idx];
        tord[tid] = idx;
    }
    __syncthreads();

    float y_one;  // NMS_YSCALE in a vector register (opaque to the compiler so it stays there)
    asm volatile("v_mov_b32 %0, 0x38800000" : "=v"(y_one));
    if (!FAST)
        small_stages<kPairExact>(tbox, taux, tord, dead1, list, flag2, wcount, n_f, part, parts, th.theta, y_one, keep_f);
    else if (scaled)
        small_stages<kPairFastYScaled>(tbox, taux, tord, dead1, list, flag2, wcount, n_f, part, parts, th.theta, y_one, keep_f);
    else
        small_stages<kPairFast>(tbox, taux, tord, dead1, list, flag2, wcount, n_f, part, parts, th.theta, y_one, keep_f);
    if (part == 0)
        for (int i = n_f + tid; i < n_max; i += kSmallThreads) keep_f[i] = 0;
}
