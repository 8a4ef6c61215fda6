// Part of nms_kernels.hip (included there, inside its anonymous namespace): the paper's rule with eliminated victims dropped from further tests, one workgroup per frame.
#pragma once

// ----------------------------------------------------------------------------- paper's rule, eliminated victims skipped

// Under the paper's rule a box survives iff NO better-ranked box eliminates it, so a victim
// that has met one eliminator needs no further test (it goes on eliminating others), and most
// victims meet theirs among the best-ranked boxes.  One workgroup (16 wavefronts) handles a
// frame.  All boxes of the frame, as outranking boxes ("candidates": box and decision
// threshold), are staged in LDS once.  The victims that are still undecided are numbered in
// rank order and cut into tiles of 64; wavefront w holds the tiles w, w + 16, w + 32, w + 48 in
// registers, lane = victim, with one wave-uniform 64-bit word per tile for the rows that are
// out.  The candidates are taken in stages [0, 128), [128, 256), [256, 512), [512, 1024),
// [1024, n): in a stage every wavefront tests its victims against the stage's candidates (read
// from LDS as broadcasts, four at a time, the next four while the current four are tested);
// after the stage the victims still alive whose rank lies beyond the stage are packed together
// (rank numbers through LDS, boxes gathered again from the table), those within it are
// survivors.  No pair is tested that involves a victim already eliminated in an earlier stage;
// nothing here depends on the order of the stages except how early victims drop out.
//
// A frame is one compute unit's work, so this route is for batches of about as many frames as
// the chip has compute units or more.  Frames of at most NMS_SORT_CHUNK boxes.
constexpr int kEarlyWaves = 16;
constexpr int kEarlyOwned = NMS_SORT_CHUNK / kTile / kEarlyWaves;  // 4
constexpr int kEarlyFirstStage = 128;   // candidates in the first stage; each further stage doubles the bound ...
constexpr int kEarlyLastBound = 1024;   // ... up to this rank, and the last stage takes the rest
constexpr int kEarlyChunk = 4;          // candidates fetched from LDS at a time

// FAST: the division-free form of nms_pair.h (the staged value per candidate is its threshold T),
// else the literal division (the staged value is its area).
template <bool FAST>
__global__ void __launch_bounds__(kEarlyWaves * 64)
early_exit_kernel(const float *__restrict__ sorted5, const int32_t *__restrict__ order,
                  const int32_t *__restrict__ counts, int n_max, int n_pad, NmsThetaConst th,
                  uint8_t *__restrict__ keep_out)
{
    __shared__ float4 cand_box_s[NMS_SORT_CHUNK];
    __shared__ float cand_aux_s[NMS_SORT_CHUNK];
    __shared__ int alive_s[NMS_SORT_CHUNK / kTile];  // packing: victims that go on, per tile
    __shared__ int ids_s[NMS_SORT_CHUNK];            // packing: their rank numbers
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
    const int staged = (n_f + kTile - 1) / kTile * kTile;  // padding rows of the table included
    for (int r = (int)threadIdx.x; r < staged; r += blockDim.x) {
        cand_box_s[r] = box4[r];
        cand_aux_s[r] = FAST ? nms_pair_threshold(area[r], th.m) : area[r];
    }

    float4 vb[kEarlyOwned];               // the victims, lane = row of the tile
    int rank_of[kEarlyOwned];             // rank number of the lane's row (0 for rows that do not exist)
    unsigned long long out[kEarlyOwned];  // wave-uniform; bit r: row r is eliminated or does not exist
    int first_rank[kEarlyOwned];          // wave-uniform: rank of the tile's first row ...
    int end_rank[kEarlyOwned];            // ... and one past the rank of its last row (both 0 for a tile that does not exist)
    int left = 0;                         // owned tiles that exist
    int n_cur = n_f;                      // victims in the current numbering

    // (re)load the owned tiles of the current numbering; `packed`: rank numbers come from ids_s
    auto load_tiles = [&](bool packed) __attribute__((always_inline)) {
        left = 0;
#pragma unroll
        for (int i = 0; i < kEarlyOwned; ++i) {
            const int first = (wave + kEarlyWaves * i) * kTile;
            const bool has = first < n_cur;
            left += has ? 1 : 0;
            const int q = first + lane;
            const bool real = q < n_cur;
            const int r = real ? (packed ? ids_s[q] : q) : 0;
            rank_of[i] = r;
            vb[i] = box4[r];
            const int rows = has ? (n_cur - first < kTile ? n_cur - first : kTile) : 0;
            out[i] = rows == kTile ? 0ull : ~0ull << rows;
            first_rank[i] = has ? __builtin_amdgcn_readlane(r, 0) : 0;
            end_rank[i] = has ? __builtin_amdgcn_readlane(r, rows - 1) + 1 : 0;
        }
    };
    load_tiles(false);
    __syncthreads();  // candidates staged, zero fill complete

    auto candidate = [&](int c, float4 &b, float &aux) __attribute__((always_inline)) {
        b = cand_box_s[c];
        aux = cand_aux_s[c];
    };
    auto hits = [&](const float4 v, const float4 cb, float aux) __attribute__((always_inline)) {
        if (FAST) return nms_eliminates_fast(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, aux);
        return nms_eliminates_exact(v.x, v.y, v.z, v.w, cb.x, cb.y, cb.z, cb.w, aux, th.theta);
    };
    // Candidates c0 .. c0+3 (already fetched) against the owned tiles.  Rank order makes the ranks
    // grow with the slot, so while the four candidates outrank the first row of slot 0 they
    // outrank every owned victim and nothing has to be checked per lane.
    auto test_chunk = [&](auto slots, const float4 (&cb)[kEarlyChunk], const float (&aux)[kEarlyChunk], int c0)
        __attribute__((always_inline)) {
        constexpr int N = decltype(slots)::value;
        if (c0 + kEarlyChunk <= first_rank[0]) {
#pragma unroll
            for (int u = 0; u < kEarlyChunk; ++u) {
#pragma unroll
                for (int i = 0; i < N; ++i) out[i] |= __ballot(hits(vb[i], cb[u], aux[u]));
            }
        } else {
#pragma unroll
            for (int i = 0; i < N; ++i) {
                if (c0 + kEarlyChunk <= first_rank[i]) {  // wave-uniform
#pragma unroll
                    for (int u = 0; u < kEarlyChunk; ++u) out[i] |= __ballot(hits(vb[i], cb[u], aux[u]));
                } else if (c0 < end_rank[i]) {
                    // the candidates' ranks run into the tile's: only better-ranked boxes eliminate
#pragma unroll
                    for (int u = 0; u < kEarlyChunk; ++u) out[i] |= __ballot(hits(vb[i], cb[u], aux[u]) && rank_of[i] > c0 + u);
                }
            }
        }
    };
    // The candidates [lo, hi) against the tiles in slots 0 .. N-1 (no further than the last owned
    // victim's rank); lo is a multiple of kEarlyChunk.
    auto run_stage = [&](auto slots, int lo, int hi) __attribute__((always_inline)) {
        constexpr int N = decltype(slots)::value;
        const int end = hi < end_rank[N - 1] ? hi : end_rank[N - 1];
        if (lo >= end) return;
        float4 box_even[kEarlyChunk], box_odd[kEarlyChunk];
        float aux_even[kEarlyChunk], aux_odd[kEarlyChunk];
#pragma unroll
        for (int u = 0; u < kEarlyChunk; ++u) candidate(lo + u, box_even[u], aux_even[u]);
        for (int c0 = lo; c0 < end; c0 += 2 * kEarlyChunk) {
            if (c0 + kEarlyChunk < end) {
#pragma unroll
                for (int u = 0; u < kEarlyChunk; ++u) candidate(c0 + kEarlyChunk + u, box_odd[u], aux_odd[u]);
            }
            test_chunk(slots, box_even, aux_even, c0);
            if (c0 + kEarlyChunk >= end) break;
            if (c0 + 2 * kEarlyChunk < end) {
#pragma unroll
                for (int u = 0; u < kEarlyChunk; ++u) candidate(c0 + 2 * kEarlyChunk + u, box_even[u], aux_even[u]);
            }
            test_chunk(slots, box_odd, aux_odd, c0 + kEarlyChunk);
        }
    };
    static_assert(kEarlyOwned == 4, "the stage dispatch below is written for up to four slots");

    int lo = 0;
    for (int bound = kEarlyFirstStage;; bound *= 2) {
        // the last stage: beyond kEarlyLastBound, or when so few victims are left that packing them
        // again would not take a tile off any wavefront
        const bool last = bound > kEarlyLastBound || bound >= n_f || n_cur <= kEarlyWaves * kTile;
        const int hi = last ? n_f : bound;
        if (left == 1) run_stage(std::integral_constant<int, 1>(), lo, hi);
        else if (left == 2) run_stage(std::integral_constant<int, 2>(), lo, hi);
        else if (left == 3) run_stage(std::integral_constant<int, 3>(), lo, hi);
        else if (left >= 4) run_stage(std::integral_constant<int, 4>(), lo, hi);
        if (last) break;

        // Victims that are alive: those ranked before `hi` have met every better-ranked box and
        // survive; the others go on, packed together.  A tile reports how many go on in
        // alive_s[tile]; a prefix sum gives every tile its place in ids_s.
        const int tiles_cur = (n_cur + kTile - 1) / kTile;
        unsigned long long on[kEarlyOwned];
#pragma unroll
        for (int i = 0; i < kEarlyOwned; ++i) {
            const bool alive = ((~out[i] >> lane) & 1ull) != 0;
            if (i < left && alive && rank_of[i] < hi) keep_f[order_f[rank_of[i]]] = 1;
            on[i] = i < left ? __ballot(alive && rank_of[i] >= hi) : 0ull;
            if (i < left && lane == 0) alive_s[wave + kEarlyWaves * i] = __builtin_popcountll(on[i]);
        }
        lds_barrier();
        const unsigned mine_alive = lane < tiles_cur ? (unsigned)alive_s[lane] : 0u;
        const unsigned incl = wave_inclusive_sum(mine_alive);
        const int total = __builtin_amdgcn_readlane((int)incl, 63);
#pragma unroll
        for (int i = 0; i < kEarlyOwned; ++i) {
            if (i < left) {  // wave-uniform
                const int base = __builtin_amdgcn_readlane((int)(incl - mine_alive), wave + kEarlyWaves * i);
                if ((on[i] >> lane) & 1ull) ids_s[base + __builtin_popcountll(on[i] & ((1ull << lane) - 1ull))] = rank_of[i];
            }
        }
        lds_barrier();
        n_cur = total;
        load_tiles(true);
        lo = hi;
    }
    // every victim still alive has met all its better-ranked boxes
#pragma unroll
    for (int i = 0; i < kEarlyOwned; ++i) {
        if (i < left && ((~out[i] >> lane) & 1ull)) keep_f[order_f[rank_of[i]]] = 1;
    }
}
