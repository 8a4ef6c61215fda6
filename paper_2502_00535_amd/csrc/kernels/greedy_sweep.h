// Part of nms_kernels.hip (included there, inside its anonymous namespace): classic greedy rule on the mask: block-wise sweep and the apply kernel between blocks.
#pragma once

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
