// Part of nms_kernels.hip (included there, inside its anonymous namespace): frames of at most 1024 boxes (a few of up to 4096), two stages of pair tests in one launch, no sort.
#pragma once

// ----------------------------------------------------------------------------- small frames, one launch

// A batch of some tens to hundreds of frames of at most a thousand boxes is too much arithmetic
// for the direct form and too little for separate launches.  Here one workgroup does everything
// for its frame, out of LDS, and nothing is sorted: Algorithm 1 asks of a pair only which of the two
// boxes is ranked first ("D[i].s < D[j].s", ties by index), and that is one compare of their
// 64-bit rank keys.  Since V_i is the AND over all j (section "Algorithm Correctness"), a victim
// that has met one eliminator needs no further test, which on clustered detections is most victims
// once some well-ranked boxes have been tried:
//
//   table     thread e holds box and key of input element e and writes row e (the box; its decision
//             threshold T, or its area for thresholds that take the literal division; the upper
//             half of its key) -- in both forms, as the box is and with y and T scaled: which one
//             the frame may use is known once every wavefront has seen its boxes, and writing
//             both lets one barrier do for the tables and that;
//   pick      the two best-ranked elements of every row of sixteen lanes (a DPP minimum over the row,
//             twice) are copied to a second table: an eighth of the frame, the best of every stretch
//             of the input -- any set of boxes would do for the result, a well-ranked one eliminates most;
//   stage 1   every victim of the workgroup against the picked boxes: lane = victim, four victims
//             per lane, the outranking boxes read from the table as broadcasts -- a broadcast moves
//             64 x 16 bytes whatever it is used for, and with one victim per lane the LDS path, not
//             the VALU, would set the pace; a box counts for the lanes whose victim is ranked
//             behind it; the compare's lane mask is the set of victims the box eliminates, ORed up
//             in a scalar register and merged per victim tile in LDS;
//   pack      victims with an eliminator are final and written out, the others are listed (box and
//             key; in the tables of the form that is not used);
//   stage 2   the listed victims against every box of the frame.  A list of up to kSmallShort
//             (clustered detections): lane = outranking box, four tiles of the table per wavefront
//             in registers, the victims read as broadcasts.  A longer list (little was
//             eliminated): the first stage's form again, with the whole table as the boxes.
//
// With fewer frames than compute units a frame is given to `parts` workgroups: each builds the
// tables of the whole frame and takes the victims of the input's tiles part, part + parts, ...  Each
// victim's keep byte is written once, by its workgroup.  Same keep vector as the all-pairs routes,
// bit for bit: a victim is dropped only once an eliminator has been found.  The kernel is held to 64
// vector registers and half a compute unit's LDS, so that two workgroups fit a compute unit.
//
// Frames of up to 2048 and 4096 boxes take the same body with two and four input elements per thread
// (mid_frames_kernel): one form of the tables, chosen after the wavefronts have exchanged their flags,
// one workgroup per compute unit, a frame shared out among up to 64 of them; for shares of one or two
// tiles the first stage takes the second stage's form (lane = outranking box, the picked boxes being
// the table).  Frames of at most 512 boxes: the body in workgroups of eight wavefronts (tiny_frames_kernel).
constexpr int kSmallWaves = 16;
constexpr int kSmallThreads = kSmallWaves * 64;
constexpr int kSmallPick = 8;                          // boxes a wavefront picks for the first stage among 64 elements
constexpr int kSmallGroup = 8;                         // outranking boxes per work item in the lane = victim form
constexpr int kSmallTiles = 4;                         // tiles a wavefront holds in registers in the second stage
constexpr int kSmallShort = 256;                       // longest list the second stage takes in its lane = outranking box form

template <int PAIR>
__device__ __forceinline__ bool small_hit(const float4 v, const float4 c, float aux, float theta, float y_one)
{
    if (PAIR == kPairFastYScaled) return nms_eliminates_fast_yscaled(v.x, v.y, v.z, v.w, c.x, c.y, c.z, c.w, aux, y_one);
    if (PAIR == kPairFast) return nms_eliminates_fast(v.x, v.y, v.z, v.w, c.x, c.y, c.z, c.w, aux);
    return nms_eliminates_exact(v.x, v.y, v.z, v.w, c.x, c.y, c.z, c.w, aux, theta);
}

__device__ __forceinline__ unsigned long long small_key(unsigned upper, int index)
{
    return ((unsigned long long)upper << 32) | (unsigned)index;
}

// The victims of a workgroup that shares its frame with others: the tiles part, part + parts, ... of the
// input (whole tiles, so that a wavefront's victims are neighbours in the table; every parts-th, so that
// an input in score order does not leave one workgroup with all the survivors).  Slot i of the share:
__device__ __forceinline__ int small_share_element(int i, int part, int parts)
{
    return ((i / kTile) * parts + part) * kTile + i % kTile;
}

// Lane = victim, one work item: the boxes [c0, c0 + kSmallGroup) of a table against R victim tiles
// (this lane's victims v[] with keys vkey[]; key 0 for a lane without a victim: nothing is ranked
// before it).  PICKED: the table of picked boxes, whose rows carry their input index; otherwise the
// frame's table, where the row number is the index.
template <int PAIR, bool PICKED, int R>
__device__ __forceinline__ void small_victim_item(const float4 *cbox, const uint4 *cinfo, const uint2 *tinfo, int c0,
                                                  const float4 (&v)[R], const unsigned long long (&vkey)[R], float theta,
                                                  float y_one, unsigned long long (&dead)[R])
{
    // four boxes at a time: with all eight in flight next to four victims' chains the kernel runs out of registers
#pragma unroll
    for (int half = 0; half < kSmallGroup; half += 4) {
        float4 cb[4];
        float ca[4];
        unsigned long long ck[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int c = c0 + half + k;
            cb[k] = cbox[c];
            if (PICKED) {
                const uint4 info = cinfo[c];
                ca[k] = __uint_as_float(info.x);
                ck[k] = small_key(info.y, (int)info.z);
            } else {
                const uint2 info = tinfo[c];
                ca[k] = __uint_as_float(info.x);
                ck[k] = small_key(info.y, c);
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
#pragma unroll
            for (int q = 0; q < R; ++q)
                dead[q] |= __ballot(small_hit<PAIR>(v[q], cb[k], ca[k], theta, y_one)) & __ballot(ck[k] < vkey[q]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
}

// Lane = victim: `count` victim slots (slot i = entry i of the list lbox / lkey; without a list, lane
// i % 64 of the workgroup's i / 64-th tile, see small_share_element; a slot at or beyond n_f holds no
// victim) in sets of R tiles against the first ncand rows (a multiple of kSmallGroup) of a table.
// The wavefronts are shared out among the sets, a wavefront keeps its set's victims in registers and takes every so-many-th group of boxes;
// eliminated victims are merged per victim tile in dead_words[].
template <int PAIR, bool PICKED, int R, int W>
__device__ __forceinline__ void small_victim_lanes(const float4 *tbox, const uint2 *tinfo, const float4 *cbox, const uint4 *cinfo,
                                                   int ncand, const float4 *lbox, const unsigned long long *lkey, int count, int n_f,
                                                   int part, int parts, unsigned long long *dead_words, float theta, float y_one)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int vtiles = (count + kTile - 1) / kTile;
    const int sets = (vtiles + R - 1) / R;  // at most 1024 / 64 / R <= 8 for R >= 2
    if (sets == 0) return;
    const int set = wave % sets;
    const int waves_of_set = (W - set + sets - 1) / sets;
    const int groups = ncand / kSmallGroup;
    float4 v[R];
    unsigned long long vkey[R];
    unsigned long long dead[R];
#pragma unroll
    for (int q = 0; q < R; ++q) {
        const int i = (R * set + q) * kTile + lane;
        if (lbox != nullptr) {
            v[q] = lbox[i < count ? i : 0];
            vkey[q] = i < count ? lkey[i] : 0ull;
        } else {
            int e = i < count ? small_share_element(i, part, parts) : -1;
            if (e >= n_f) e = -1;
            v[q] = tbox[e < 0 ? 0 : e];
            vkey[q] = e < 0 ? 0ull : small_key(tinfo[e].y, e);
        }
        dead[q] = 0ull;
    }
    for (int g = wave / sets; g < groups; g += waves_of_set)
        small_victim_item<PAIR, PICKED, R>(cbox, cinfo, tinfo, g * kSmallGroup, v, vkey, theta, y_one, dead);
    if (lane == 0) {
#pragma unroll
        for (int q = 0; q < R; ++q)
            if (dead[q] != 0ull) atomicOr(&dead_words[R * set + q], dead[q]);
    }
}

// Lane = outranking box: `count` victim slots (entry i of the list lbox / lkey; without a list, slot i of the
// workgroup's share, see small_share_element) against the first ctiles tiles of a table.  A wavefront
// keeps one group of TILES tiles in registers and takes every so-many-th batch of four victims, read as
// broadcasts, their reads issued together (a slot beyond the count repeats the last one); a victim with
// an eliminator gets its bit in dead_words[slot / 64].  PICKED: the table of picked boxes, whose rows
// carry their input index; otherwise the frame's table, where the row number is the index.
template <int PAIR, bool PICKED, int TILES, int W>
__device__ __forceinline__ void small_candidate_lanes(const float4 *tbox, const uint2 *tinfo, const float4 *cbox, const uint4 *cinfo,
                                                      int ctiles, const float4 *lbox, const unsigned long long *lkey, int count,
                                                      int n_f, int part, int parts, unsigned long long *dead_words, float theta,
                                                      float y_one)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int groups = (ctiles + TILES - 1) / TILES;
    const int batches = (count + 3) / 4;
    if (groups == 0 || batches == 0) return;
    const int g = wave % groups;
    const int waves_of_group = (W - g + groups - 1) / groups;
    const int first_batch = wave / groups;
    if (first_batch >= batches) return;
    float4 cb[TILES];
    float aux[TILES];
    unsigned long long ckey[TILES];
#pragma unroll 1
    for (int t0 = g * TILES; t0 < ctiles; t0 += W * TILES) {  // (more groups than wavefronts: the table of a long frame)
#pragma unroll
        for (int j = 0; j < TILES; ++j) {
            const bool real = t0 + j < ctiles;  // a tile beyond the table's last: a copy of tile t0 that is ranked before nothing
            const int row = (t0 + (real ? j : 0)) * kTile + lane;
            cb[j] = cbox[row];
            if (PICKED) {
                const uint4 info = cinfo[row];
                aux[j] = __uint_as_float(info.x);
                ckey[j] = real ? small_key(info.y, (int)info.z) : ~0ull;
            } else {
                const uint2 info = tinfo[row];
                aux[j] = __uint_as_float(info.x);
                ckey[j] = real ? small_key(info.y, row) : ~0ull;
            }
        }
#pragma unroll 1
        for (int batch = first_batch; batch < batches; batch += waves_of_group) {
            int at[4];
            float4 v[4];
            unsigned long long vkey[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                at[u] = 4 * batch + u < count ? 4 * batch + u : count - 1;
                if (lbox != nullptr) {
                    v[u] = lbox[at[u]];
                    vkey[u] = lkey[at[u]];
                } else {
                    const int e = small_share_element(at[u], part, parts);
                    v[u] = tbox[e < n_f ? e : 0];
                    vkey[u] = e < n_f ? small_key(tinfo[e].y, e) : 0ull;  // no victim in this slot: nothing is ranked before key 0
                }
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                unsigned long long any = 0ull;
#pragma unroll
                for (int j = 0; j < TILES; ++j)
                    any |= __ballot(small_hit<PAIR>(v[u], cb[j], aux[j], theta, y_one)) & __ballot(ckey[j] < vkey[u]);
                if (lane == 0 && any != 0ull) atomicOr(&dead_words[at[u] / kTile], 1ull << (at[u] % kTile));
            }
        }
    }
}

// The stages of one workgroup.  tbox / tinfo: the frame in input order (info = decision value, upper
// key half); pbox / pinfo: the picked boxes (info = decision value, upper key half, input index).  The
// workgroup's victims are the slots i < m0 of its share (small_share_element).
template <int PAIR, int PICK_TILES, int W>
__device__ __forceinline__ void small_stages(const float4 *tbox, const uint2 *tinfo, const float4 *pbox, const uint4 *pinfo,
                                             int picked_rows, unsigned long long *dead1, unsigned long long *dead2, float4 *lbox,
                                             unsigned long long *lkey, int n_f, int part, int parts, float theta, float y_one,
                                             uint8_t *keep_f)
{
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tiles_f = (n_f + kTile - 1) / kTile;
    const int m0 = tiles_f > part ? (tiles_f - part + parts - 1) / parts * kTile : 0;  // victim slots of the share

    // ---- stage 1: lane = victim, four victims per lane, where the share has three tiles or more (a broadcast of an
    // outranking box then serves four rows), two per lane for two tiles; lane = outranking box for a single tile
    if (m0 / kTile > 2)
        small_victim_lanes<PAIR, true, 4, W>(tbox, tinfo, pbox, pinfo, picked_rows, nullptr, nullptr, m0, n_f, part, parts, dead1, theta, y_one);
    else if (m0 / kTile == 2 && PICK_TILES == 2)
        small_victim_lanes<PAIR, true, 2, W>(tbox, tinfo, pbox, pinfo, picked_rows, nullptr, nullptr, m0, n_f, part, parts, dead1, theta, y_one);
    else
        small_candidate_lanes<PAIR, true, PICK_TILES, W>(tbox, tinfo, pbox, pinfo, picked_rows / kTile, nullptr, nullptr, m0, n_f, part, parts,
                                                         dead1, theta, y_one);
    __syncthreads();

    // ---- pack: victims with an eliminator are written out, the others listed (box and key), in slot order.  How many
    // each of the share's tiles lists follows from dead1[], which every wavefront sums up for itself (lane t: tile t; a
    // DPP prefix sum inside rows of sixteen lanes) -- no exchange of counts, no barrier for it.
    const int t_lane = lane & 15;
    int in_tile = n_f - (t_lane * parts + part) * kTile;  // victims in tile t_lane of the share
    in_tile = t_lane * kTile < m0 ? (in_tile < 0 ? 0 : (in_tile > kTile ? kTile : in_tile)) : 0;
    const unsigned long long there = in_tile >= kTile ? ~0ull : (1ull << in_tile) - 1ull;
    const int sums = (int)row16_inclusive_sum((unsigned)__popcll(there & ~dead1[t_lane]));
    const int listed = __builtin_amdgcn_readlane(sums, 15);
    const int before = wave == 0 ? 0 : __builtin_amdgcn_readlane(sums, wave - 1);
    bool alive = false;
    int e_mine = 0;
    if (tid < m0 && small_share_element(tid, part, parts) < n_f) {
        e_mine = small_share_element(tid, part, parts);
        if (((dead1[wave] >> lane) & 1ull) != 0ull)
            keep_f[e_mine] = 0;
        else
            alive = true;
    }
    const unsigned long long alive_mask = __ballot(alive);
    if (alive) {
        const int pos = before + (int)__builtin_amdgcn_mbcnt_hi((unsigned)(alive_mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)alive_mask, 0u));
        lbox[pos] = tbox[e_mine];
        lkey[pos] = small_key(tinfo[e_mine].y, e_mine);
    }
    __syncthreads();

    // ---- stage 2: the listed victims against the whole frame
    if (listed <= kSmallShort)
        small_candidate_lanes<PAIR, false, kSmallTiles, W>(tbox, tinfo, tbox, nullptr, tiles_f, lbox, lkey, listed, n_f, 0, 1, dead2, theta, y_one);
    if (listed > kSmallShort)
        small_victim_lanes<PAIR, false, 4, W>(tbox, tinfo, tbox, nullptr, tiles_f * kTile, lbox, lkey, listed, n_f, 0, 1, dead2, theta, y_one);
    __syncthreads();
    for (int k = tid; k < listed; k += W * kTile) keep_f[(unsigned)lkey[k]] = ((dead2[k / kTile] >> (k % kTile)) & 1ull) != 0ull ? 0 : 1;
}

// The kernel's body.  W: wavefronts of the workgroup (T = 64 W threads); E: input elements per thread
// (frames of at most E * T boxes); register q of thread t holds element T q + t, so a wavefront's
// register is a tile of 64 neighbours.  A workgroup's share is at most T victims.  FAST: the threshold
// has a division-free form (NmsThetaConst).
template <bool FAST, int E, int W>
__device__ __forceinline__ void small_frames_body(const float *__restrict__ boxes, const float *__restrict__ scores,
                                                  const int32_t *__restrict__ counts, int n_max, int parts, const NmsThetaConst &th,
                                                  uint8_t *__restrict__ keep_out)
{
    constexpr int T = W * kTile;               // threads of the workgroup
    constexpr int P = T * E;                   // rows of the tables
    constexpr int kPicked = W * kSmallPick * E;  // rows of the table of picked boxes
    // One element per thread: every table twice, as the boxes are and with y (and the decision value) multiplied by
    // NMS_YSCALE -- which of the two the stages read is known only once every wavefront has seen its boxes, and
    // writing both saves a barrier; the list of the second stage then takes the place of the form that is not used.
    // Longer frames have no room for that: the wavefronts exchange their flags first and write one form.
    constexpr int kForms = (FAST && E == 1) ? 2 : 1;
    constexpr int kList = kForms == 2 ? 1 : T;  // a workgroup's share is at most one victim per thread
    __shared__ float4 tbox[kForms][P];
    __shared__ uint2 tinfo[kForms][P];
    __shared__ float4 pbox[kForms][kPicked];
    __shared__ uint4 pinfo[kForms][kPicked];
    __shared__ unsigned long long dead1[16];
    __shared__ unsigned long long dead2[16];
    __shared__ float4 lbox_own[kList];
    __shared__ unsigned long long lkey_own[kList];
    __shared__ int wodd[W];
    const int f = blockIdx.x / parts;
    const int part = blockIdx.x % parts;
    const int tid = (int)threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int n_f = frame_count(counts, f, n_max);
    const float *scores_f = scores + (size_t)f * n_max;
    const float4 *boxes_f = reinterpret_cast<const float4 *>(boxes + (size_t)f * n_max * 4);
    uint8_t *keep_f = keep_out + (size_t)f * n_max;

    // a slot beyond the frame's count holds the box (0,0,0,0) with the last of all keys: it is ranked before no
    // box of the frame
    float4 mine[E];
    unsigned upper[E];
#pragma unroll
    for (int q = 0; q < E; ++q) {
        const int e = q * T + tid;
        mine[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        upper[q] = ~0u;
        if (e < n_f) {
            mine[q] = boxes_f[e];
            upper[q] = (unsigned)(nms_rank_key(scores_f[e], (unsigned)e) >> 32);
        }
    }
    // pick: the two best-ranked elements of every row of sixteen lanes (equal upper key halves: the lower lane first)
    bool picked[E];
    int slot[E];
    bool odd = false;
#pragma unroll
    for (int q = 0; q < E; ++q) {
        picked[q] = false;
#pragma unroll
        for (int round = 0; round < kSmallPick / 4; ++round) {
            const unsigned u = picked[q] ? ~0u : upper[q];
            const unsigned best = row16_min(u);
            const unsigned long long is_best = __ballot(u == best && !picked[q]);
            const unsigned in_row = (unsigned)(is_best >> (lane & 48)) & 0xffffu;
            if (u == best && !picked[q] && (in_row & ((1u << (lane & 15)) - 1u)) == 0u) picked[q] = true;
        }
        const unsigned long long picked_mask = __ballot(picked[q]);
        slot[q] = (q * W + wave) * kSmallPick +
                  (int)__builtin_amdgcn_mbcnt_hi((unsigned)(picked_mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)picked_mask, 0u));
        // per frame: does every y allow the scaled form (the box (0,0,0,0) does)
        odd = odd || !(nms_y_regular(mine[q].y) && nms_y_regular(mine[q].w));
    }
    const unsigned long long odd_mask = __ballot(odd);
    if (lane == 0) wodd[wave] = odd_mask != 0ull ? 1 : 0;
    if (tid < 16) {
        dead1[tid] = 0ull;
        dead2[tid] = 0ull;
    }
    bool scaled = false;
    if (kForms == 1 && FAST) {
        __syncthreads();
        scaled = __ballot(wodd[lane & (W - 1)] != 0) == 0ull;
    }
    // what the tables need per box: its decision value (no intersection reaches a padding row's)
#pragma unroll
    for (int q = 0; q < E; ++q) {
        const int e = q * T + tid;
        const float area = nms_box_area(mine[q].x, mine[q].y, mine[q].z, mine[q].w);
        const float aux = FAST ? (e < n_f ? nms_pair_threshold(area, th.m) : INFINITY) : area;
        const float y1 = mine[q].y, y2 = mine[q].w;
        const float4 mine_s = make_float4(mine[q].x, y1 * NMS_YSCALE, mine[q].z, y2 * NMS_YSCALE);
        const float aux_s = aux * NMS_YSCALE;
        const bool first_scaled = kForms == 1 && scaled;  // the only form is the scaled one
        const float4 row = make_float4(mine[q].x, first_scaled ? mine_s.y : y1, mine[q].z, first_scaled ? mine_s.w : y2);
        const float row_aux = first_scaled ? aux_s : aux;
        tbox[0][e] = row;
        tinfo[0][e] = make_uint2(__float_as_uint(row_aux), upper[q]);
        if (picked[q]) {
            pbox[0][slot[q]] = row;
            pinfo[0][slot[q]] = make_uint4(__float_as_uint(row_aux), upper[q], (unsigned)e, 0u);
        }
        if (kForms == 2) {
            tbox[kForms - 1][e] = mine_s;
            tinfo[kForms - 1][e] = make_uint2(__float_as_uint(aux_s), upper[q]);
            if (picked[q]) {
                pbox[kForms - 1][slot[q]] = mine_s;
                pinfo[kForms - 1][slot[q]] = make_uint4(__float_as_uint(aux_s), upper[q], (unsigned)e, 0u);
            }
        }
    }
    __syncthreads();
    if (kForms == 2) scaled = __ballot(wodd[lane & (W - 1)] != 0) == 0ull;

    float y_one;  // NMS_YSCALE in a vector register (opaque to the compiler so it stays there)
    asm volatile("v_mov_b32 %0, 0x38800000" : "=v"(y_one));
    constexpr int kPickTiles = kPicked / kTile < kSmallTiles ? kPicked / kTile : kSmallTiles;  // tiles of picked boxes a wavefront holds when the boxes are the lanes
    if (!FAST)
        small_stages<kPairExact, kPickTiles, W>(tbox[0], tinfo[0], pbox[0], pinfo[0], kPicked, dead1, dead2, lbox_own, lkey_own, n_f, part,
                                             parts, th.theta, y_one, keep_f);
    else if (kForms == 1 && scaled)
        small_stages<kPairFastYScaled, kPickTiles, W>(tbox[0], tinfo[0], pbox[0], pinfo[0], kPicked, dead1, dead2, lbox_own, lkey_own, n_f,
                                                   part, parts, th.theta, y_one, keep_f);
    else if (kForms == 1)
        small_stages<kPairFast, kPickTiles, W>(tbox[0], tinfo[0], pbox[0], pinfo[0], kPicked, dead1, dead2, lbox_own, lkey_own, n_f, part,
                                            parts, th.theta, y_one, keep_f);
    else if (scaled)
        small_stages<kPairFastYScaled, kPickTiles, W>(tbox[kForms - 1], tinfo[kForms - 1], pbox[kForms - 1], pinfo[kForms - 1], kPicked,
                                                   dead1, dead2, tbox[0], reinterpret_cast<unsigned long long *>(tinfo[0]), n_f, part,
                                                   parts, th.theta, y_one, keep_f);
    else
        small_stages<kPairFast, kPickTiles, W>(tbox[0], tinfo[0], pbox[0], pinfo[0], kPicked, dead1, dead2, tbox[kForms - 1],
                                            reinterpret_cast<unsigned long long *>(tinfo[kForms - 1]), n_f, part, parts, th.theta,
                                            y_one, keep_f);
    if (part == 0)
        for (int i = n_f + tid; i < n_max; i += T) keep_f[i] = 0;
}

// Frames of at most 1024 boxes.  Grid: frames * parts workgroups of kSmallThreads threads.  Held to
// eight wavefronts per SIMD: two workgroups per compute unit.
template <bool FAST>
__global__ void __launch_bounds__(kSmallThreads) __attribute__((amdgpu_waves_per_eu(8, 8)))
small_frames_kernel(const float *__restrict__ boxes, const float *__restrict__ scores, const int32_t *__restrict__ counts,
                    int n_max, int parts, NmsThetaConst th, uint8_t *__restrict__ keep_out)
{
    small_frames_body<FAST, 1, kSmallWaves>(boxes, scores, counts, n_max, parts, th, keep_out);
}

// Frames of at most 1024 E boxes, E = 2 or 4; a workgroup's share is at most 1024 victims (parts >= tiles / 16).
template <bool FAST, int E>
__global__ void __launch_bounds__(kSmallThreads) __attribute__((amdgpu_waves_per_eu(4, 4)))
mid_frames_kernel(const float *__restrict__ boxes, const float *__restrict__ scores, const int32_t *__restrict__ counts,
                  int n_max, int parts, NmsThetaConst th, uint8_t *__restrict__ keep_out)
{
    small_frames_body<FAST, E, kSmallWaves>(boxes, scores, counts, n_max, parts, th, keep_out);
}

// Frames of at most 512 boxes: workgroups of eight wavefronts, up to four of them on a compute unit.
constexpr int kTinyWaves = 8;
constexpr int kTinyThreads = kTinyWaves * 64;
template <bool FAST>
__global__ void __launch_bounds__(kTinyThreads) __attribute__((amdgpu_waves_per_eu(8, 8)))
tiny_frames_kernel(const float *__restrict__ boxes, const float *__restrict__ scores, const int32_t *__restrict__ counts,
                   int n_max, int parts, NmsThetaConst th, uint8_t *__restrict__ keep_out)
{
    small_frames_body<FAST, 1, kTinyWaves>(boxes, scores, counts, n_max, parts, th, keep_out);
}
