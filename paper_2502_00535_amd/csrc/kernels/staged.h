// Part of nms_kernels.hip (included there, inside its anonymous namespace): the paper's rule on large frames in two launches, decided victims dropped in between.
#pragma once

// ----------------------------------------------------------------------------- large frames, two launches

// A victim is decided by its first eliminator (section "Algorithm Correctness": V_i is the AND
// over all j), and on clustered detections most victims meet theirs among the best-ranked boxes.
// For a frame too large for one workgroup's LDS the same idea runs at the scale of the grid:
//
//   first launch   every victim against the best kStageTiles * 64 ranks only -- the fused map
//                  kernel's pair loop (lane = victim, outranking box through scalar loads), one
//                  64 x 64 tile per wavefront.  Each unit clears keep_out for the victims it
//                  eliminates and leaves their lane mask in dead_part[victim tile][outranking tile].
//   second launch  the victims still alive (one in eight on a dense crowd scene) are numbered in
//                  rank order from the masks, and a wavefront takes 64 CONSECUTIVE LIVE victims --
//                  not a tile of 64 ranks -- against the remaining outranking tiles up to the rank
//                  of its last victim, one tile per work unit.  Tiles that reach into the
//                  ranks of the wavefront's own victims mask every lane by "outranking box ranked
//                  before my victim".  The workgroups are persistent and share the units out by
//                  stride; the tables that turn a unit number into (victims, tiles) are a few
//                  prefix sums in LDS, rebuilt by every workgroup from the masks.
//
// Same keep vector as the all-pairs kernel, bit for bit: a victim is dropped only once an
// eliminator has been found, and every other pair is tested by the same instructions.
constexpr int kStageTiles = 32;   // outranking tiles of the first launch: the best 2048 ranks (1024: its 7 us against 11, but 26 us for the second launch against 13)
constexpr int kStageSplit = 1;    // work units per outranking tile in the second launch (2: 15 us instead of 13; a unit's set-up costs more than its tile)
constexpr int kStageWaves = 16;   // wavefronts per workgroup of the second launch
constexpr int kStageMaxTiles = NMS_MAX_N / NMS_TILE;

// Position of the n-th set bit of m (n counted from 0; n < popcount(m)).
__device__ __forceinline__ int nth_set_bit(unsigned long long m, int n)
{
    int pos = 0;
#pragma unroll
    for (int w = 32; w >= 1; w >>= 1) {
        const unsigned long long low = m & ((1ull << w) - 1ull);
        const int c = __popcll(low);
        if (n >= c) {
            n -= c;
            m >>= w;
            pos += w;
        } else {
            m = low;
        }
    }
    return pos;
}

// Largest i in [0, count) with table[i] <= x, for an ascending table with table[0] <= x.
__device__ __forceinline__ int last_not_above(const int *table, int count, int x)
{
    int lo = 0, hi = count - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (table[mid] <= x) lo = mid;
        else hi = mid - 1;
    }
    return lo;
}

// Exclusive prefix sums of table[0 .. count) in place, table[count] = total; run by one wavefront.
__device__ __forceinline__ void wave_exclusive_scan(int *table, int count, int lane)
{
    const int per = (count + 63) / 64;  // consecutive entries per lane
    const int first = lane * per;
    int sum = 0;
    for (int i = first; i < first + per && i < count; ++i) sum += table[i];
    const int before = (int)wave_inclusive_sum((unsigned)sum) - sum;
    int run = before;
    for (int i = first; i < first + per && i < count; ++i) {
        const int v = table[i];
        table[i] = run;
        run += v;
    }
    const int total = __builtin_amdgcn_readlane((int)wave_inclusive_sum((unsigned)sum), 63);
    if (lane == 0) table[count] = total;
}

// First launch.  Unit g = (victim tile tr, outranking tile tc) with tc < kStageTiles, tc <= tr;
// the four wavefronts of a workgroup share a victim tile.
template <bool FAST>
__global__ void __launch_bounds__(kMapWaves * 64)
staged_first_kernel(const float *__restrict__ sorted5, const int32_t *__restrict__ counts, int n_max, int n_pad,
                    NmsThetaConst th, const int32_t *__restrict__ order, uint8_t *__restrict__ keep_out,
                    const float4 *__restrict__ ysc, const unsigned *__restrict__ ytile, const float *__restrict__ tsc,
                    unsigned long long *__restrict__ dead_part)
{
    const int lane = threadIdx.x & 63;
    const int f = blockIdx.y;
    const int g = __builtin_amdgcn_readfirstlane((int)blockIdx.x * kMapWaves + (int)(threadIdx.x >> 6));
    const int T = n_pad / kTile;
    const int tr = g / kStageTiles;
    const int tc = g % kStageTiles;
    const int n_f = frame_count(counts, f, n_max);
    const int tiles_f = (n_f + kTile - 1) / kTile;
    if (tr >= tiles_f || tc > tr) return;

    const float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    const float4 *__restrict__ box4 = reinterpret_cast<const float4 *>(sorted_f);
    const float *__restrict__ area = sorted_f + 4 * (size_t)n_pad;
    const float4 *__restrict__ ysc4 = ysc + (size_t)f * n_pad;
    const unsigned *__restrict__ ytile_f = ytile + (size_t)f * (n_pad / kTile);
    const float *__restrict__ tsc_f = tsc + (size_t)f * n_pad;
    float y_one;  // NMS_YSCALE in a vector register (opaque to the compiler so it stays there)
    asm volatile("v_mov_b32 %0, 0x38800000" : "=v"(y_one));

    const int row = tr * kTile + lane;
    unsigned long long acc;
    if (FAST && ytile_f[tr] != 0 && ytile_f[tc] != 0) {
        const float4 vbs = ysc4[row];
        if (tc == tr)
            acc = fused_candidates<kPairFastYScaled, kMaskDiagonal>(ysc4 + tc * kTile, tsc_f + tc * kTile, vbs, y_one, th.theta, 0, 0);
        else
            acc = fused_candidates<kPairFastYScaled, kMaskNone>(ysc4 + tc * kTile, tsc_f + tc * kTile, vbs, y_one, th.theta, 0, 0);
    } else {
        const float4 vb = box4[row];
        const float *caux = FAST ? tsc_f + tc * kTile : area + tc * kTile;
        if (tc == tr)
            acc = fused_candidates<FAST ? kPairFast : kPairExact, kMaskDiagonal>(box4 + tc * kTile, caux, vb, y_one, th.theta, 0, 0);
        else
            acc = fused_candidates<FAST ? kPairFast : kPairExact, kMaskNone>(box4 + tc * kTile, caux, vb, y_one, th.theta, 0, 0);
    }
    if (lane == 0) dead_part[((size_t)f * T + tr) * kStageTiles + tc] = acc;
    if (((acc >> lane) & 1ull) && row < n_f) keep_out[(size_t)f * n_max + order[(size_t)f * n_max + row]] = 0;
}

struct StagedShared {
    unsigned long long alive[kStageMaxTiles];  // per tile of ranks: victims that no box of the first launch eliminated
    int before[kStageMaxTiles + 1];            // live victims ranked before tile t; [T] = all of them
    int units[kStageMaxTiles + 1];             // work units before the s-th run of 64 live victims; [runs] = all of them
};

// Second launch: gridDim.x persistent workgroups per frame.
template <bool FAST>
__global__ void __launch_bounds__(kStageWaves * 64)
staged_second_kernel(const float *__restrict__ sorted5, const int32_t *__restrict__ counts, int n_max, int n_pad,
                     NmsThetaConst th, const int32_t *__restrict__ order, uint8_t *__restrict__ keep_out,
                     const float4 *__restrict__ ysc, const unsigned *__restrict__ ytile, const float *__restrict__ tsc,
                     const unsigned long long *__restrict__ dead_part)
{
    __shared__ StagedShared sh;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int f = blockIdx.y;
    const int T = n_pad / kTile;
    const int n_f = frame_count(counts, f, n_max);
    const int tiles_f = (n_f + kTile - 1) / kTile;
    if (tiles_f <= kStageTiles) return;  // every victim met all its outranking boxes in the first launch (uniform)

    // the victims still alive, per tile of ranks; tiles below kStageTiles are settled.  Four
    // neighbouring lanes share a tile: a quarter of its masks each, all loads in flight together.
    for (int q = tid; q < 4 * T; q += kStageWaves * 64) {  // 4 T and the thread count are multiples of 64
        const int t = q >> 2;
        const bool open = t >= kStageTiles && t < tiles_f;
        unsigned long long dead = 0;
        if (open) {
            constexpr int kPer = kStageTiles / 4;
            const unsigned long long *part = dead_part + ((size_t)f * T + t) * kStageTiles + kPer * (q & 3);
            unsigned long long d[kPer];
#pragma unroll
            for (int c = 0; c < kPer; ++c) d[c] = part[c];
#pragma unroll
            for (int c = 0; c < kPer; ++c) dead |= d[c];
        }
        dead |= __shfl_xor(dead, 1);
        dead |= __shfl_xor(dead, 2);
        if ((q & 3) == 0) {
            unsigned long long m = 0;
            if (open) {
                const int in_tile = n_f - t * kTile;  // boxes of the frame in this tile (>= 1)
                const unsigned long long real = in_tile >= kTile ? ~0ull : ((1ull << in_tile) - 1ull);
                m = ~dead & real;
            }
            sh.alive[t] = m;
            sh.before[t] = __popcll(m);
        }
    }
    __syncthreads();
    if (wave == 0) wave_exclusive_scan(sh.before, T, lane);
    __syncthreads();
    const int A = sh.before[T];       // live victims
    const int runs = (A + 63) / 64;   // a wavefront takes a run of 64 consecutive live victims
    if (A == 0) return;               // uniform

    // rank of the a-th live victim
    auto rank_of = [&](int a) -> int {
        const int t = last_not_above(sh.before, T, a);
        return t * kTile + nth_set_bit(sh.alive[t], a - sh.before[t]);
    };
    // work units of run s: the outranking tiles kStageTiles .. (tile of its last victim), kStageSplit units per tile
    for (int s = tid; s < runs; s += kStageWaves * 64) {
        const int last = 64 * s + 63 < A ? 64 * s + 63 : A - 1;
        const int top = rank_of(last) / kTile;
        sh.units[s] = (top - kStageTiles + 1) * kStageSplit;
    }
    __syncthreads();
    if (wave == 0) wave_exclusive_scan(sh.units, runs, lane);
    __syncthreads();
    const int U = sh.units[runs];

    const float *sorted_f = sorted5 + (size_t)f * 5 * n_pad;
    const float4 *__restrict__ box4 = reinterpret_cast<const float4 *>(sorted_f);
    const float *__restrict__ area = sorted_f + 4 * (size_t)n_pad;
    const float4 *__restrict__ ysc4 = ysc + (size_t)f * n_pad;
    const unsigned *__restrict__ ytile_f = ytile + (size_t)f * (n_pad / kTile);
    const float *__restrict__ tsc_f = tsc + (size_t)f * n_pad;
    float y_one;
    asm volatile("v_mov_b32 %0, 0x38800000" : "=v"(y_one));

    const int stride = (int)gridDim.x * kStageWaves;
    for (int u = (int)blockIdx.x * kStageWaves + wave; u < U; u += stride) {  // u is wave-uniform
        const int s = last_not_above(sh.units, runs, u);
        const int piece = u - sh.units[s];
        const int a = 64 * s + lane;
        const bool active = a < A;
        const int r = active ? rank_of(a) : 0;      // this lane's victim (rank order along the lanes)
        const int mine = active ? r : -1;            // never ranked behind anything when the lane is idle
        const int last_lane = 64 * s + 63 < A ? 63 : A - 1 - 64 * s;
        const int lo_tile = __builtin_amdgcn_readfirstlane(r) / kTile;              // lane 0 is always active
        const int top = __builtin_amdgcn_readlane(r, last_lane) / kTile;
        const int tc = kStageTiles + piece / kStageSplit;  // <= top: run s has (top - kStageTiles + 1) * kStageSplit units

        const float4 vbs = ysc4[r];
        const float4 vb = box4[r];
        const bool v_regular = FAST && __ballot(active && !(nms_y_regular(vb.y) && nms_y_regular(vb.w))) == 0ull;
        unsigned long long acc;
        const bool masked = tc >= lo_tile;  // the tile reaches into the ranks of this run's own victims
        if (v_regular && ytile_f[tc] != 0) {
            if (masked)
                acc = fused_candidates_ahead<kPairFastYScaled, kMaskByRank>(ysc4 + tc * kTile, tsc_f + tc * kTile, vbs, y_one,
                                                                            th.theta, mine, tc * kTile);
            else
                acc = fused_candidates_ahead<kPairFastYScaled, kMaskNone>(ysc4 + tc * kTile, tsc_f + tc * kTile, vbs, y_one,
                                                                          th.theta, mine, tc * kTile);
        } else {
            const float *caux = FAST ? tsc_f + tc * kTile : area + tc * kTile;
            if (masked)
                acc = fused_candidates<FAST ? kPairFast : kPairExact, kMaskByRank>(box4 + tc * kTile, caux, vb, y_one, th.theta,
                                                                                   mine, tc * kTile);
            else
                acc = fused_candidates<FAST ? kPairFast : kPairExact, kMaskNone>(box4 + tc * kTile, caux, vb, y_one, th.theta,
                                                                                 mine, tc * kTile);
        }
        if (active && ((acc >> lane) & 1ull)) keep_out[(size_t)f * n_max + order[(size_t)f * n_max + r]] = 0;
    }
}
